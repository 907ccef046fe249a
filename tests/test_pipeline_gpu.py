"""GPU: the producer->consumer ring (Section 3.3) delivers every minibatch bit-exactly, in order,
with a slow consumer and with a consumer that is ahead, and refuses to overwrite a held buffer."""
import numpy as np
import pytest

import zcg_workload as wl
from oracle import gather as oracle_gather

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
z = pytest.importorskip("paper_2103_03330_amd")
from paper_2103_03330_amd import probe  # noqa: E402


@pytest.mark.parametrize("n_buffers,masked,slow_consumer", [(2, False, False), (2, True, True),
                                                            (3, False, True), (1, False, False)])
def test_ring_delivers_every_minibatch(n_buffers, masked, slow_consumer):
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    torch.cuda.set_device(0)
    n_rows, dim = 50_000, 100
    table = z.alloc_table(n_rows, dim, "f32")
    wl.fill_table_ptr(table.host_ptr, n_rows, dim, "f32", seed=31)
    g = wl.PowerLawGraph(n_rows, 20.0, 2.1, seed=5)
    lists = [g.sample_minibatch(64, (10, 5), b)[0] for b in range(12)] + [np.zeros(0, np.int64)]
    g.close()
    max_rows = max(a.size for a in lists)
    bufs = [torch.zeros((max_rows, dim), dtype=torch.float32, device="cuda") for _ in range(n_buffers)]
    gstream = z.stream_create_cu_mask(list(range(16))) if masked else None
    pipe = z.pipeline_create(table, max_rows, bufs, gstream)
    consumer = torch.cuda.Stream()
    sink = torch.zeros(256, dtype=torch.float32, device="cuda")
    results = []
    torch.cuda.synchronize()
    try:
        pending = []  # slots submitted and not yet consumed, in order
        for b, idx in enumerate(lists):
            if len(pending) == n_buffers:  # ring full: consume the oldest first
                slot, want_rows = pending.pop(0)
                buf, n = pipe.acquire(slot, consumer)
                assert n == want_rows
                with torch.cuda.stream(consumer):
                    if slow_consumer:
                        probe.synthetic_compute(consumer, 2048, 20000, sink)
                    results.append(buf[:n].clone())
                pipe.release(slot, consumer)
            pending.append((pipe.submit(idx), idx.size))
        while pending:
            slot, want_rows = pending.pop(0)
            buf, n = pipe.acquire(slot, consumer)
            with torch.cuda.stream(consumer):
                results.append(buf[:n].clone())
            pipe.release(slot, consumer)
        consumer.synchronize()
        assert len(results) == len(lists)
        host = table.host_array()
        for b, (idx, got) in enumerate(zip(lists, results)):
            want = oracle_gather(host, idx)
            assert got.cpu().numpy().tobytes() == want.tobytes(), f"minibatch {b}"
        # a buffer that was submitted but not released cannot be overwritten
        for _ in range(n_buffers):
            s = pipe.submit(lists[0])
        with pytest.raises(z.ZcgError) as e:
            pipe.submit(lists[1])
        assert e.value.status == z.binding.EBUSY
        with pytest.raises(z.ZcgError) as e:
            pipe.submit(np.array([n_rows]))
        assert e.value.status == z.binding.ERANGE
    finally:
        pipe.close()
        if gstream:
            gstream.close()
        table.close()


def test_producer_thread_and_consumer_thread():
    """The paper's arrangement: a producer (sampler + gather) and a consumer run side by side and
    meet through a bounded queue. Here they are two host threads on the ring's blocking calls."""
    import threading

    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    torch.cuda.set_device(0)
    n_rows, dim, n_batches, n_buffers = 80_000, 100, 30, 2
    table = z.alloc_table(n_rows, dim, "f32")
    wl.fill_table_ptr(table.host_ptr, n_rows, dim, "f32", seed=41)
    g = wl.PowerLawGraph(n_rows, 25.0, 2.1, seed=9)
    max_rows = 128 * 11 * 6
    bufs = [torch.zeros((max_rows, dim), dtype=torch.float32, device="cuda") for _ in range(n_buffers)]
    pipe = z.pipeline_create(table, max_rows, bufs)
    submitted, results, errors = [], [], []

    def producer():
        try:
            torch.cuda.set_device(0)
            for b in range(n_batches):
                idx = g.sample_minibatch(128, (10, 5), b)[0]
                submitted.append(idx)
                pipe.submit(idx, timeout_ms=20_000)
            pipe.finish()
        except Exception as exc:  # noqa: BLE001
            errors.append(("producer", repr(exc)))
            pipe.finish()

    def consumer():
        try:
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()
            sink = torch.zeros(256, dtype=torch.float32, device="cuda")
            while True:
                slot = pipe.next(timeout_ms=20_000)
                if slot is None:
                    break
                buf, n = pipe.acquire(slot, stream)
                with torch.cuda.stream(stream):
                    probe.synthetic_compute(stream, 512, 4000, sink)  # the consumer is the slower side
                    results.append(buf[:n].clone())
                pipe.release(slot, stream)
            stream.synchronize()
        except Exception as exc:  # noqa: BLE001
            errors.append(("consumer", repr(exc)))

    tp, tc = threading.Thread(target=producer), threading.Thread(target=consumer)
    try:
        tc.start()
        tp.start()
        tp.join(timeout=100)
        tc.join(timeout=100)
        assert not tp.is_alive() and not tc.is_alive()
        assert not errors, errors
        assert len(results) == n_batches == len(submitted)
        host = table.host_array()
        for b, (idx, got) in enumerate(zip(submitted, results)):
            assert got.cpu().numpy().tobytes() == oracle_gather(host, idx).tobytes(), f"minibatch {b}"
        # after finish: the producer is refused, the consumer is told the stream has ended
        with pytest.raises(z.ZcgError) as e:
            pipe.submit(submitted[0])
        assert e.value.status == z.ECLOSED
        assert pipe.next(timeout_ms=0) is None
    finally:
        torch.cuda.synchronize()
        pipe.close()
        g.close()
        table.close()


def test_bounded_waits_time_out():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    torch.cuda.set_device(0)
    n_rows, dim = 10_000, 64
    table = z.alloc_table(n_rows, dim, "f16")
    wl.fill_table_ptr(table.host_ptr, n_rows, dim, "f16", seed=43)
    bufs = [torch.zeros((100, dim), dtype=torch.float16, device="cuda")]
    pipe = z.pipeline_create(table, 100, bufs)
    try:
        with pytest.raises(z.ZcgError) as e:
            pipe.next(timeout_ms=30)  # nothing submitted
        assert e.value.status == z.ETIMEDOUT
        idx = np.arange(100, dtype=np.int64)
        slot = pipe.submit(idx)
        with pytest.raises(z.ZcgError) as e:
            pipe.submit(idx, timeout_ms=30)  # the only buffer is held
        assert e.value.status == z.ETIMEDOUT
        with pytest.raises(z.ZcgError) as e:
            pipe.submit(idx)
        assert e.value.status == z.EBUSY
        assert pipe.next(timeout_ms=0) == slot
        buf, n = pipe.acquire(slot)
        torch.cuda.synchronize()
        assert n == 100 and buf[:n].cpu().numpy().tobytes() == oracle_gather(table.host_array(), idx).tobytes()
        pipe.release(slot)
        with pytest.raises(z.ZcgError) as e:
            pipe.release(slot)  # already released
        assert e.value.status == z.binding.EINVAL
        assert pipe.submit(idx, timeout_ms=30) == 0
    finally:
        torch.cuda.synchronize()
        pipe.close()
        table.close()


def test_ring_sorts_short_rows_by_itself():
    """Tables with rows of at most a line: lists that are long and dense enough in the table
    (here the 150,001-entry ones) are gathered in ascending table order inside the ring, short
    ones in list order; the delivered rows are in list order either way."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    torch.cuda.set_device(0)
    for dim, dtype, tdt in ((16, "f16", torch.float16), (32, "f32", torch.float32), (5, "f32", torch.float32)):
        n_rows = 200_000
        table = z.alloc_table(n_rows, dim, dtype)
        wl.fill_table_ptr(table.host_ptr, n_rows, dim, dtype, seed=47 + dim)
        lists = [wl.uniform_indices(n, n_rows, seed=n) for n in (150_001, 1, 33_333, 150_001)]
        bufs = [torch.zeros((150_001, dim), dtype=tdt, device="cuda") for _ in range(2)]
        pipe = z.pipeline_create(table, 150_001, bufs)
        try:
            for idx in lists:
                slot = pipe.submit(idx)
                buf, n = pipe.acquire(slot)
                torch.cuda.synchronize()
                assert n == idx.size
                assert buf[:n].cpu().numpy().tobytes() == oracle_gather(table.host_array(), idx).tobytes()
                pipe.release(slot)
        finally:
            torch.cuda.synchronize()
            pipe.close()
            table.close()


@pytest.mark.parametrize("extra_rows", [0, 4096])
def test_lists_cross_the_link_narrow_up_to_2_32_rows_and_wide_beyond(extra_rows):
    """Row numbers of a table of at most 2^32 rows are staged and copied as 32-bit values and widened
    on the GPU (the largest, 2^32 - 1, included); one more row and the list travels as int64."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    torch.cuda.set_device(0)
    n_rows = (1 << 32) + extra_rows
    table = z.alloc_table(n_rows, 1, "i8")  # 4.3 GB of one-byte rows
    try:
        host = table.host_array()
        rng = np.random.default_rng(77 + extra_rows)
        regions = [(0, 5000), ((1 << 31) - 3000, (1 << 31) + 3000), (n_rows - 6000, n_rows)]
        parts = []
        for lo, hi in regions:
            host[lo:hi, 0] = rng.integers(-128, 128, hi - lo, dtype=np.int8)
            parts.append(rng.integers(lo, hi, 4000, dtype=np.int64))
        parts.append(np.array([0, n_rows - 1, (1 << 32) - 1, 1 << 31], dtype=np.int64))
        idx = rng.permutation(np.concatenate(parts))
        bufs = [torch.zeros((idx.size, 1), dtype=torch.int8, device="cuda") for _ in range(2)]
        pipe = z.pipeline_create(table, idx.size, bufs)
        try:
            for lst in (idx, idx[::-1].copy(), idx[:1]):
                slot = pipe.submit(lst)
                buf, n = pipe.acquire(slot)
                torch.cuda.synchronize()
                assert n == lst.size
                assert buf[:n].cpu().numpy().tobytes() == oracle_gather(host, lst).tobytes()
                pipe.release(slot)
            with pytest.raises(Exception):
                pipe.submit(np.array([n_rows], dtype=np.int64))
        finally:
            torch.cuda.synchronize()
            pipe.close()
    finally:
        table.close()
