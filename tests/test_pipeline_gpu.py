"""GPU: the producer->consumer ring (Section 3.3) delivers every minibatch bit-exactly, in order,
with a slow consumer and with a consumer that is ahead, and refuses to overwrite a held buffer."""
import numpy as np
import pytest

import zcg_workload as wl
from oracle import gather as oracle_gather

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
z = pytest.importorskip("paper_2103_03330_amd")


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
                        z.synthetic_compute(consumer, 2048, 20000, sink)
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
