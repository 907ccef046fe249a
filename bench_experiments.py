"""The secondary experiments of bench.py (``--config 5 ... 12``): width/dtype sweep, alignment
sweep, resource provisioning, producer/consumer pipeline, list-length sweep, the fixed launch
sequence behind the link's request model, the request rate against table size and the HBM-resident
variant against a plain device copy. The headline path (configs 1-4) stays in bench.py.

Every function takes the parsed arguments and the modules bench.py has already imported
(``z`` = paper_2103_03330_amd, ``wl`` = zcg_workload, numpy, torch) and returns plain data that
bench.py prints as one JSON line. ``probe`` is paper_2103_03330_amd.probe."""
from __future__ import annotations

import sys
import time

from paper_2103_03330_amd import probe

PEAK_NOTE = ("above 1: the peak is the copy engine's measured rate over the same link, the metric's "
             "denominator, not a ceiling; GPU-issued reads stream slightly faster, and rows a list "
             "repeats are served from the GPU's L2")


def build_workload(z, wl, k, n_batches, flags, max_table_gb):
    cfg = wl.config(k)
    n_rows = cfg.n_rows
    note = None
    if cfg.table_bytes > max_table_gb * 1e9:
        n_rows = int(max_table_gb * 1e9 // cfg.row_bytes // 1_000_000 * 1_000_000)
        note = f"table scaled to {n_rows} rows to fit host memory"
    t0 = time.time()
    table = z.alloc_table(n_rows, cfg.dim, cfg.dtype, flags)
    wl.fill_table_ptr(table.host_ptr, n_rows, cfg.dim, cfg.dtype, cfg.seed)
    t_table = time.time() - t0
    t0 = time.time()
    if cfg.graph is None:
        lists = [wl.uniform_indices(cfg.n_idx, n_rows, (cfg.seed ^ 0x1D) + b) for b in range(n_batches)]
    else:
        g = wl.PowerLawGraph(n_rows, cfg.graph[0], cfg.graph[1], cfg.seed)
        lists = [g.sample_minibatch(cfg.n_seeds, cfg.fanout, b)[0] for b in range(n_batches)]
        g.close()
    return cfg, table, lists, dict(table_s=round(t_table, 2), sampler_s=round(time.time() - t0, 2),
                                   note=note, n_rows=n_rows)


def run_sweep(args, z, wl, np, torch, link_peak):
    """Config 5: 10 M rows x dim in {16,64,256,1024}, fp16 and fp32, 1 M uniform indices per call;
    host-resident zero-copy vs the same table copied to HBM, and the DMA method. Every leg cycles
    over 8 distinct lists, as training would (no leg sees the same rows twice in a row, so neither
    the GPU's L2 nor the CPU's last-level cache is warmed by the previous call). One JSON line."""
    points = []
    n_lists = 8
    for cfg in wl.sweep_configs():
        if args.only_point and cfg.name != args.only_point:
            continue
        table = z.alloc_table(cfg.n_rows, cfg.dim, cfg.dtype)
        wl.fill_table_ptr(table.host_ptr, cfg.n_rows, cfg.dim, cfg.dtype, cfg.seed)
        lists = [wl.uniform_indices(cfg.n_idx, cfg.n_rows, (cfg.seed ^ 0x1D) + b) for b in range(n_lists)]
        idx_dev = [torch.from_numpy(a).cuda() for a in lists]
        n = cfg.n_idx
        tdt = torch.float32 if cfg.dtype == "f32" else torch.float16
        out = torch.empty((n, cfg.dim), dtype=tdt, device="cuda")
        stream = torch.cuda.current_stream()
        reps = max(8, min(args.steps, 24))

        def timed(call):
            """Median time of call(b) over `reps` calls that cycle through the lists."""
            for b in range(3):
                call(b)
            torch.cuda.synchronize()
            ms = []
            for i in range(reps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                call((3 + i) % n_lists)
                e1.record(stream)
                e1.synchronize()
                ms.append(e0.elapsed_time(e1))
            return float(np.median(ms))

        useful = n * cfg.row_bytes
        # zcg_gather: rows walked in list order
        ms_list = timed(lambda b: z.gather_variant(table, idx_dev[b], out, args.variant, stream=stream))
        # the default call with workspace lent: AUTO walks short rows in ascending table order
        # when that pays, building the order itself inside the timed call
        ws_bytes = z.gather_workspace_bytes(n)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        lent = z.LaunchOpts(variant=args.variant, workspace_dev=ws.data_ptr(), workspace_bytes=ws_bytes)
        ms_host = timed(lambda b: z.gather_ex(table, idx_dev[b], out, lent, stream=stream))
        ms_ord = None
        if cfg.row_bytes <= 128:  # the orders built beforehand (what a caller who reuses lists pays)
            orders = [torch.empty(n, dtype=torch.int64, device="cuda") for _ in range(n_lists)]
            for b in range(n_lists):
                z.make_order(idx_dev[b], cfg.n_rows, orders[b], ws, ws_bytes, stream=stream)
            ms_ord = timed(lambda b: z.gather_ordered(table, idx_dev[b], orders[b], out, stream=stream))
            del orders
        del ws
        hbm_t = torch.empty((cfg.n_rows, cfg.dim), dtype=tdt, device="cuda")
        host = table.host_array()
        step = max(1, (1 << 30) // cfg.row_bytes)
        for lo in range(0, cfg.n_rows, step):
            hbm_t[lo:lo + step].copy_(torch.from_numpy(host[lo:lo + step]))
        t2 = z.table_from_device(hbm_t, cfg.n_rows, cfg.dim, cfg.dtype)
        ms_hbm = timed(lambda b: z.gather_variant(t2, idx_dev[b], out, args.variant, stream=stream))
        t2.close()
        del hbm_t
        staging = z.pinned_alloc(useful)
        dma_runs = {}
        for name, fn in (("one_shot", lambda b: z.cpu_gather_memcpy(table, lists[b], staging, out,
                                                                   wl.default_threads(), stream)),
                         ("chunked", lambda b: z.cpu_gather_memcpy_chunked(
                             table, lists[b], staging, out, max(1024, (4 << 20) // cfg.row_bytes),
                             wl.default_threads(), stream))):
            fn(0)  # warm-up: first touch of the staging pages
            torch.cuda.synchronize()
            t = []
            for i in range(n_lists):
                t0 = time.perf_counter()
                fn((i + 1) % n_lists)
                torch.cuda.synchronize()
                t.append(time.perf_counter() - t0)
            dma_runs[name] = useful / float(np.median(t)) / 1e9
        dma = max(dma_runs.values())
        z.pinned_free(staging)
        lines = -(-cfg.row_bytes // 128)
        points.append({"name": cfg.name, "row_bytes": cfg.row_bytes,
                       "zero_copy_gbps": round(useful / ms_host / 1e6, 2),
                       "fraction_of_link_peak": round(useful / ms_host / 1e6 / link_peak, 4),
                       "rows_per_s": round(n / ms_host * 1e3),
                       "call": "zcg_gather_ex, variant AUTO, workspace lent",
                       "list_order_gbps": round(useful / ms_list / 1e6, 2),
                       "order_built_beforehand_gbps": round(useful / ms_ord / 1e6, 2) if ms_ord else None,
                       "peak_note": PEAK_NOTE if useful / ms_host / 1e6 > link_peak else None,
                       "useful_over_line_bytes": round(cfg.row_bytes / (lines * 128), 3),
                       "hbm_resident_gbps": round(useful / ms_hbm / 1e6, 1),
                       "dma_baseline_gbps": round(dma, 2),
                       "dma_one_shot_gbps": round(dma_runs["one_shot"], 2),
                       "dma_chunked_gbps": round(dma_runs["chunked"], 2),
                       "zero_copy_speedup": round(useful / ms_host / 1e6 / dma, 3)})
        table.close()
        print(f"# {points[-1]}", file=sys.stderr, flush=True)
    return points


def run_align_sweep(args, z, wl, np, torch, link_peak):
    """The paper's Section 4.2 experiment (its Figure 8) on synthetic data: rows of 1024...1044 bytes
    (fp32 dim 256...261) in a 13.6 M-row table, sampled index lists; every kernel and the DMA method."""
    n_rows, points = 13_600_000, []
    g = wl.PowerLawGraph(n_rows, 32.0, 2.1, wl.MASTER_SEED + 6)
    lists = [g.sample_minibatch(1024, (15, 10), b)[0] for b in range(8)]
    g.close()
    idx_dev = [torch.from_numpy(a).cuda() for a in lists]
    stream = torch.cuda.current_stream()
    for dim in range(256, 262):
        rb = dim * 4
        table = z.alloc_table(n_rows, dim, "f32")
        wl.fill_table_ptr(table.host_ptr, n_rows, dim, "f32", wl.MASTER_SEED + 6)
        out = torch.empty((max(a.size for a in lists), dim), dtype=torch.float32, device="cuda")
        pt = {"row_bytes": rb}
        for name, variant in (("naive", z.VARIANT_NAIVE), ("rowvec", z.VARIANT_ROWVEC),
                              ("aligned", z.VARIANT_ALIGNED), ("halfline", z.VARIANT_HALFLINE),
                              ("auto", z.VARIANT_AUTO)):
            for b in range(2):
                z.gather_variant(table, idx_dev[b], out, variant, stream=stream)
            torch.cuda.synchronize()
            tot_ms, rows = 0.0, 0
            for i in range(max(8, min(args.steps, 40))):
                b = i % len(lists)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                z.gather_variant(table, idx_dev[b], out, variant, stream=stream)
                e1.record(stream)
                e1.synchronize()
                tot_ms += e0.elapsed_time(e1)
                rows += lists[b].size
            pt[name + "_gbps"] = round(rows * rb / tot_ms / 1e6, 2)
            pt[name + "_frac"] = round(rows * rb / tot_ms / 1e6 / link_peak, 4)
        staging = z.pinned_alloc(out.numel() * 4)
        for name, fn in (("dma_one_shot_gbps", lambda b: z.cpu_gather_memcpy(
                              table, lists[b], staging, out, wl.default_threads(), stream)),
                         ("dma_chunked_gbps", lambda b: z.cpu_gather_memcpy_chunked(
                              table, lists[b], staging, out, max(1024, (4 << 20) // rb),
                              wl.default_threads(), stream))):
            fn(len(lists) - 1)  # warm-up: first touch of the staging pages
            torch.cuda.synchronize()
            t0, rows = time.perf_counter(), 0
            for b in range(len(lists)):
                fn(b)
                torch.cuda.synchronize()
                rows += lists[b].size
            pt[name] = round(rows * rb / (time.perf_counter() - t0) / 1e9, 2)
        z.pinned_free(staging)
        pt["plan_auto"] = z.VARIANT_NAMES[z.plan_gather(table, lists[0].size, out)["variant"]]
        table.close()
        points.append(pt)
        print(f"# {pt}", file=sys.stderr, flush=True)
    return points, int(np.mean([a.size for a in lists]))


def run_provisioning(args, z, wl, np, torch, link_peak):
    """Section 3.2.2 / 4.3 of the paper on one MI355X: how much of the GPU the gather needs, and what
    capping its share buys when compute kernels run beside it. The share is set by binding the
    gather's stream to a subset of the compute units (the paper used a process-level service)."""
    cfg, table, lists, _ = build_workload(z, wl, 2, 16, z.ALLOC_DEFAULT, args.max_table_gb)
    rb = cfg.row_bytes
    idx_dev = [torch.from_numpy(a).cuda() for a in lists]
    outs = [torch.empty((max(a.size for a in lists), cfg.dim), dtype=torch.float32, device="cuda")
            for _ in range(2)]
    n_cus = z.device_cu_count(0)
    reps = max(16, min(args.steps, 64))

    def spread(n):
        # bit i of the mask is compute unit i/8 of accelerator die i%8: the first n bits, n a
        # multiple of 8, take n/8 compute units on each of the 8 dies (the runtime refuses a
        # mask that leaves a die without any)
        return list(range(n))

    def gather_rate(stream_obj, opts=None):
        ts = torch.cuda.ExternalStream(stream_obj.cuda_stream) if hasattr(stream_obj, "cu_ids") else stream_obj
        for i in range(3):
            z.gather_ex(table, idx_dev[i % 16], outs[i & 1], opts, n_idx=lists[i % 16].size, stream=ts)
        ts.synchronize()
        tot, rows = 0.0, 0
        for i in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(ts)
            z.gather_ex(table, idx_dev[i % 16], outs[i & 1], opts, n_idx=lists[i % 16].size, stream=ts)
            e1.record(ts)
            e1.synchronize()
            tot += e0.elapsed_time(e1)
            rows += lists[i % 16].size
        return rows * rb / tot / 1e6

    share_curve = []
    for n in (8, 16, 24, 32, 40, 64, 128, 256):
        n = min(n, n_cus)
        ms = z.stream_create_cu_mask(spread(n))
        g = gather_rate(ms)
        ms.close()
        share_curve.append({"cus": n, "share_percent": round(100.0 * n / n_cus, 1), "gbps": round(g, 2),
                            "fraction_of_link_peak": round(g / link_peak, 4)})
        print(f"# {share_curve[-1]}", file=sys.stderr, flush=True)
    grid_curve = []
    cur = torch.cuda.current_stream()
    for blocks in (4, 8, 16, 32, 64, 128, 256, 2048):
        g = gather_rate(cur, z.LaunchOpts(max_blocks=blocks))
        grid_curve.append({"blocks": blocks, "waves": blocks * 4, "gbps": round(g, 2),
                           "fraction_of_link_peak": round(g / link_peak, 4)})
        print(f"# {grid_curve[-1]}", file=sys.stderr, flush=True)

    # overlap with a compute kernel that fills the GPU: per minibatch one gather + one compute
    sink = torch.zeros(256, dtype=torch.float32, device="cuda")
    comp_blocks = n_cus * 64  # many short blocks: no tail when some compute units are masked off
    iters = 4000
    probe.synthetic_compute(cur, comp_blocks, iters, sink)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        probe.synthetic_compute(cur, comp_blocks, iters, sink)
    torch.cuda.synchronize()
    per = (time.perf_counter() - t0) / 5
    iters = max(1000, int(iters * 2.0e-3 / per))  # about 2 ms alone: twice one gather

    def minibatch_ms(gs, cs, same_stream=False):
        for s_ in {gs, cs}:
            s_.synchronize()
        t = time.perf_counter()
        for i in range(reps):
            z.gather_ex(table, idx_dev[i % 16], outs[i & 1], None, n_idx=lists[i % 16].size, stream=gs)
            probe.synthetic_compute(cs if not same_stream else gs, comp_blocks, iters, sink)
        gs.synchronize()
        cs.synchronize()
        return (time.perf_counter() - t) / reps * 1e3

    probe.synthetic_compute(cur, comp_blocks, iters, sink)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        probe.synthetic_compute(cur, comp_blocks, iters, sink)
    torch.cuda.synchronize()
    compute_alone = (time.perf_counter() - t0) / reps * 1e3
    gather_alone = float(np.mean([a.size for a in lists])) * rb / gather_rate(cur) / 1e6
    overlap = [{"mode": "one stream (serial)", "ms_per_minibatch": round(minibatch_ms(cur, cur, True), 3)}]
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    overlap.append({"mode": "two streams, no masks", "ms_per_minibatch": round(minibatch_ms(s1, s2), 3)})
    for n in (8, 16, 24, 40, 64, 128):
        n = min(n, n_cus - 8)
        gcu = spread(n)
        ccu = [c for c in range(n_cus) if c not in set(gcu)]
        mg, mc = z.stream_create_cu_mask(gcu), z.stream_create_cu_mask(ccu)
        tg, tc = torch.cuda.ExternalStream(mg.cuda_stream), torch.cuda.ExternalStream(mc.cuda_stream)
        overlap.append({"mode": f"masks {n}:{n_cus - n} CUs ({100.0 * n / n_cus:.1f}% gather)",
                        "ms_per_minibatch": round(minibatch_ms(tg, tc), 3)})
        mg.close()
        mc.close()
        print(f"# {overlap[-1]}", file=sys.stderr, flush=True)
    table.close()
    rtt_us = probe.measure_host_read_latency(20000)
    full = share_curve[-1]["gbps"]
    lines_per_s = full * 1e9 / rb * 4  # a 400-byte row costs four 128-byte lines
    littles = {"host_read_round_trip_us": round(rtt_us, 3),
               "lines_per_s_at_full_rate": round(lines_per_s),
               "lines_in_flight": round(lines_per_s * rtt_us * 1e-6),
               "bytes_in_flight": round(lines_per_s * rtt_us * 1e-6 * 128),
               "note": "Little's law with the unloaded round trip: a lower bound on what must be in flight"}
    print(f"# {littles}", file=sys.stderr, flush=True)
    return {"littles_law": littles, "gather_vs_cu_share": share_curve, "gather_vs_grid_size": grid_curve,
            "overlap": {"gather_alone_ms": round(gather_alone, 3), "compute_alone_ms": round(compute_alone, 3),
                        "compute_blocks": comp_blocks, "compute_iters": iters, "cases": overlap}}


def run_pipeline(args, z, wl, np, torch, link_peak):
    """Section 3.3 of the paper on one MI355X: sampler -> producer (list copy + gather) -> consumer
    (a synthetic compute kernel standing in for training) with two alternating GPU buffers and one
    event hand-off per minibatch, against the same work done step by step on one stream."""
    cfg, table, lists, _ = build_workload(z, wl, 2, 16, z.ALLOC_DEFAULT, args.max_table_gb)
    rb, n_cus = cfg.row_bytes, z.device_cu_count(0)
    max_rows = max(a.size for a in lists)
    reps = max(32, min(args.steps, 128))
    sink = torch.zeros(256, dtype=torch.float32, device="cuda")
    comp_blocks, iters = n_cus * 64, 6000  # about 2 ms on the whole GPU
    bufs = [torch.empty((max_rows, cfg.dim), dtype=torch.float32, device="cuda") for _ in range(2)]
    cur = torch.cuda.current_stream()

    # step by step on one stream: copy list, gather, compute, wait
    idx_dev = torch.empty(max_rows, dtype=torch.int64, device="cuda")
    pinned = [torch.from_numpy(a).pin_memory() for a in lists]

    def serial_step(i):
        a = pinned[i % 16]
        idx_dev[:a.numel()].copy_(a, non_blocking=True)
        z.gather(table, idx_dev, bufs[0], n_idx=a.numel(), stream=cur)
        probe.synthetic_compute(cur, comp_blocks, iters, sink)
        torch.cuda.synchronize()

    only = args.pipeline_mode  # run one mode only (for kernel-trace profiles)
    serial_ms = None
    if only in ("all", "serial"):
        for i in range(3):
            serial_step(i)
        t0 = time.perf_counter()
        for i in range(reps):
            serial_step(i)
        serial_ms = (time.perf_counter() - t0) / reps * 1e3

    def pipelined(gather_cus):
        if gather_cus:
            gs = z.stream_create_cu_mask(list(range(gather_cus)))
            cs = z.stream_create_cu_mask(list(range(gather_cus, n_cus)))
            cons = torch.cuda.ExternalStream(cs.cuda_stream)
        else:
            gs, cs, cons = None, None, torch.cuda.Stream()
        pipe = z.pipeline_create(table, max_rows, bufs, gs)
        torch.cuda.synchronize()
        t = time.perf_counter()
        prev = None
        for i in range(reps + 1):
            slot = pipe.submit(lists[i % 16]) if i < reps else None  # producer runs one ahead
            if prev is not None:
                pipe.acquire(prev, cons)
                probe.synthetic_compute(cons, comp_blocks, iters, sink)
                pipe.release(prev, cons)
            prev = slot
        cons.synchronize()
        ms = (time.perf_counter() - t) / reps * 1e3
        pipe.close()
        if gs:
            gs.close()
            cs.close()
        return ms

    def ring_alone(n_buffers):
        """Nothing but the ring: the consumer takes each buffer and lets go of it at once, so the
        gather bounds the loop and whatever the ring adds to the kernel's own time shows."""
        rb_bufs = bufs if n_buffers == 2 else bufs + [torch.empty_like(bufs[0]) for _ in range(n_buffers - 2)]
        cons = torch.cuda.Stream()
        pipe = z.pipeline_create(table, max_rows, rb_bufs, None)
        for i in range(n_buffers):  # warm-up: every slot used once
            s0 = pipe.submit(lists[i % 16])
            pipe.acquire(s0, cons)
            pipe.release(s0, cons)
        torch.cuda.synchronize()
        t = time.perf_counter()
        pending = []
        for i in range(reps):
            pending.append(pipe.submit(lists[i % 16], timeout_ms=10_000))
            if len(pending) == n_buffers:
                s0 = pending.pop(0)
                pipe.acquire(s0, cons)
                pipe.release(s0, cons)
        for s0 in pending:
            pipe.acquire(s0, cons)
            pipe.release(s0, cons)
        cons.synchronize()
        ms = (time.perf_counter() - t) / reps * 1e3
        pipe.close()
        return ms

    # The same with the sampler inside the loop (Section 3.3: sampling, gathering and training are
    # three stages; the first two run beside the third). Lists are drawn live from the graph.
    def sampler_graph():
        return wl.PowerLawGraph(table.n_rows, cfg.graph[0], cfg.graph[1], cfg.seed)

    bound_rows = cfg.n_seeds
    for f in cfg.fanout:
        bound_rows *= f + 1

    def serial_with_sampler():
        g = sampler_graph()
        big = torch.empty((bound_rows, cfg.dim), dtype=torch.float32, device="cuda")
        idx_big = torch.empty(bound_rows, dtype=torch.int64, device="cuda")
        t_s = 0.0
        torch.cuda.synchronize()
        t = time.perf_counter()
        for b in range(reps):
            ts = time.perf_counter()
            a = torch.from_numpy(g.sample_minibatch(cfg.n_seeds, cfg.fanout, b)[0])
            t_s += time.perf_counter() - ts
            idx_big[:a.numel()].copy_(a, non_blocking=False)
            z.gather(table, idx_big, big, n_idx=a.numel(), stream=cur)
            probe.synthetic_compute(cur, comp_blocks, iters, sink)
            torch.cuda.synchronize()
        ms = (time.perf_counter() - t) / reps * 1e3
        g.close()
        return ms, t_s / reps * 1e3

    def threaded(gather_cus, n_samplers=1):
        import queue
        import threading
        g = sampler_graph()
        lists_q = queue.Queue(maxsize=2 * n_samplers)
        counter, counter_lock = [0], threading.Lock()

        def sampler():  # several samplers feed one producer, as the paper's sampler workers do
            mine = sampler_graph()  # a graph object carries its own visited-bitmap: one per thread
            try:
                while True:
                    with counter_lock:
                        b = counter[0]
                        counter[0] += 1
                    if b >= reps:
                        return
                    lists_q.put(mine.sample_minibatch(cfg.n_seeds, cfg.fanout, b)[0])
            finally:
                mine.close()
        tbufs = [torch.empty((bound_rows, cfg.dim), dtype=torch.float32, device="cuda") for _ in range(2)]
        if gather_cus:
            gs = z.stream_create_cu_mask(list(range(gather_cus)))
            cs = z.stream_create_cu_mask(list(range(gather_cus, n_cus)))
            cons = torch.cuda.ExternalStream(cs.cuda_stream)
        else:
            gs, cs, cons = None, None, torch.cuda.Stream()
        pipe = z.pipeline_create(table, bound_rows, tbufs, gs)
        failed = []

        def producer():
            try:
                torch.cuda.set_device(0)
                for b in range(reps):
                    a = (lists_q.get(timeout=60) if n_samplers > 1
                         else g.sample_minibatch(cfg.n_seeds, cfg.fanout, b)[0])
                    pipe.submit(a, timeout_ms=60_000)
            except Exception as exc:  # noqa: BLE001
                failed.append(repr(exc))
            finally:
                pipe.finish()

        def consumer():
            try:
                torch.cuda.set_device(0)
                while True:
                    slot = pipe.next(timeout_ms=60_000)
                    if slot is None:
                        break
                    pipe.acquire(slot, cons)
                    probe.synthetic_compute(cons, comp_blocks, iters, sink)
                    pipe.release(slot, cons)
                cons.synchronize()
            except Exception as exc:  # noqa: BLE001
                failed.append(repr(exc))

        tp, tc = threading.Thread(target=producer), threading.Thread(target=consumer)
        samplers = [threading.Thread(target=sampler) for _ in range(n_samplers if n_samplers > 1 else 0)]
        torch.cuda.synchronize()
        t = time.perf_counter()
        for th in samplers + [tc, tp]:
            th.start()
        for th in samplers + [tp, tc]:
            th.join()
        ms = (time.perf_counter() - t) / reps * 1e3
        pipe.close()
        if gs:
            gs.close()
            cs.close()
        g.close()
        if failed:
            raise RuntimeError(f"threaded pipeline failed: {failed}")
        return ms

    cases = []
    if serial_ms is not None:
        cases.append({"mode": "one stream, step by step", "ms_per_minibatch": round(serial_ms, 3)})
    if only in ("all", "threads"):
        ms, sample_ms = serial_with_sampler()
        cases.append({"mode": "sampler in the loop, one stream, step by step", "ms_per_minibatch": round(ms, 3),
                      "sampler_ms": round(sample_ms, 3)})
        cases.append({"mode": "sampler+producer thread | consumer thread, 2 buffers, no masks",
                      "ms_per_minibatch": round(threaded(0), 3)})
        cases.append({"mode": f"sampler+producer thread | consumer thread, 2 buffers, gather on 16 CUs / compute on {n_cus - 16}",
                      "ms_per_minibatch": round(threaded(16), 3)})
        cases.append({"mode": f"4 sampler threads -> producer thread | consumer thread, 2 buffers, gather on 16 CUs / compute on {n_cus - 16}",
                      "ms_per_minibatch": round(threaded(16, 4), 3)})
    if only in ("all", "ring"):
        rows_avg = float(np.mean([lists[i % 16].size for i in range(reps)]))
        for nb in (2, 3):
            ms = ring_alone(nb)
            cases.append({"mode": f"ring alone (no consumer work), {nb} buffers", "ms_per_minibatch": round(ms, 4),
                          "gathered_GBps": round(rows_avg * rb / ms / 1e6, 2)})
    if only in ("all", "nomask"):
        cases.append({"mode": "pipeline, 2 buffers, no masks", "ms_per_minibatch": round(pipelined(0), 3)})
    for n in (8, 16, 24):
        if only in ("all", f"mask{n}"):
            cases.append({"mode": f"pipeline, 2 buffers, gather on {n} CUs / compute on {n_cus - n}",
                          "ms_per_minibatch": round(pipelined(n), 3)})
    probe.synthetic_compute(cur, comp_blocks, iters, sink)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        probe.synthetic_compute(cur, comp_blocks, iters, sink)
    torch.cuda.synchronize()
    compute_ms = (time.perf_counter() - t0) / reps * 1e3
    table.close()
    for c in cases:
        print(f"# {c}", file=sys.stderr, flush=True)
    return {"compute_alone_ms": round(compute_ms, 3), "rows_per_minibatch_avg": float(np.mean([a.size for a in lists])),
            "cases": cases}


def run_request_blocks(args, z, wl, np, torch):
    """Which unit the link's read requests come in: random rows of 128 ... 512 bytes (row pitch =
    row size) read from a mapped base that is a multiple of 256 bytes, then from the same base
    plus 128 bytes, with the launch shape of host-resident tables in both cases."""
    n_rows, n_idx = 4_000_000, 400_000
    cur = torch.cuda.current_stream()
    pts = []
    for dim in (128, 96, 64, 32):
        rb = dim * 4
        base = z.alloc_table(n_rows + 2, dim, "f32")
        idx = torch.from_numpy(wl.uniform_indices(n_idx, n_rows, seed=5)).cuda()
        out = torch.empty((n_idx, dim), dtype=torch.float32, device="cuda")
        for off in (0, 128):
            view = z.table_from_device(base.device_ptr + off, n_rows, dim, "f32")
            o = z.LaunchOpts(unroll=2, nt_loads=2, max_blocks=2048 if rb > 128 else 8192,
                             vec_bytes=8 if rb > 128 else 16, group_lanes=64 if rb > 128 else 16)
            for _ in range(3):
                z.gather_ex(view, idx, out, o, stream=cur)
            torch.cuda.synchronize()
            ms = []
            for _ in range(20):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(cur)
                z.gather_ex(view, idx, out, o, stream=cur)
                e1.record(cur)
                e1.synchronize()
                ms.append(e0.elapsed_time(e1))
            t = float(np.median(ms))
            pts.append({"row_bytes": rb, "base_offset": off, "gbps": round(n_idx * rb / t / 1e6, 2),
                        "rows_per_s": round(n_idx / t * 1e3)})
            print(f"# {pts[-1]}", file=sys.stderr, flush=True)
            view.close()
        if rb == 256:
            # the same rows fetched one 128-byte line per load instruction (64 lanes x 2 bytes), with
            # one or two such loads in flight: do the two lines of a pair have to share an instruction?
            view = z.table_from_device(base.device_ptr, n_rows, rb, "i8")
            out8 = out.view(torch.int8).view(n_idx, rb)
            for in_flight in (1, 2):
                o = z.LaunchOpts(variant=z.VARIANT_ROWVEC, unroll=in_flight, nt_loads=2, max_blocks=8192,
                                 vec_bytes=2, group_lanes=64)
                for _ in range(3):
                    z.gather_ex(view, idx, out8, o, stream=cur)
                torch.cuda.synchronize()
                ms = []
                for _ in range(20):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(cur)
                    z.gather_ex(view, idx, out8, o, stream=cur)
                    e1.record(cur)
                    e1.synchronize()
                    ms.append(e0.elapsed_time(e1))
                t = float(np.median(ms))
                pts.append({"row_bytes": rb, "base_offset": 0, "gbps": round(n_idx * rb / t / 1e6, 2),
                            "rows_per_s": round(n_idx / t * 1e3),
                            "loads": f"one line per instruction, {in_flight} in flight per wave"})
                print(f"# {pts[-1]}", file=sys.stderr, flush=True)
            view.close()
        base.close()
    return pts


def run_request_sequence(args, z, wl, np, torch):
    """A fixed sequence of gathers, each configuration launched 4 times in a row (the first is a
    warm-up), for matching rocprofv3 per-dispatch counters and kernel-trace durations to
    configurations by order: the kernels of config 2 at full and at capped grid sizes (how many
    reads must be in flight), and random rows of 128 ... 512 bytes on and off the 256-byte grid
    (what the link counts as one request). Prints the labels in launch order."""
    labels, reps = [], 4

    def run(label, table, idx_dev, out, opts, n, rb):
        for _ in range(reps):
            z.gather_ex(table, idx_dev, out, opts, n_idx=n)
            torch.cuda.synchronize()
        labels.append({"label": label, "n_idx": int(n), "row_bytes": int(rb), "launches": reps})

    cfg = wl.config(2)
    table = z.alloc_table(cfg.n_rows, cfg.dim, cfg.dtype)
    wl.fill_table_ptr(table.host_ptr, cfg.n_rows, cfg.dim, cfg.dtype, cfg.seed)
    idx = wl.index_lists(cfg)[0]
    idx_dev = torch.from_numpy(idx).cuda()
    out = torch.empty((idx.size, cfg.dim), dtype=torch.float32, device="cuda")
    seq = [("cfg2 rowvec", dict(variant=z.VARIANT_ROWVEC)), ("cfg2 aligned", dict(variant=z.VARIANT_ALIGNED)),
           ("cfg2 half-all", dict(variant=z.VARIANT_HALFLINE, half_ends=1)),
           ("cfg2 half-lone", dict(variant=z.VARIANT_HALFLINE, half_ends=2))]
    seq += [(f"cfg2 half-lone {b} blocks", dict(variant=z.VARIANT_HALFLINE, half_ends=2, max_blocks=b))
            for b in (8, 16, 32, 48, 64, 96, 128, 256, 1024, 4096)]
    seq += [(f"cfg2 aligned {b} blocks", dict(variant=z.VARIANT_ALIGNED, max_blocks=b)) for b in (16, 32, 64, 128, 256)]
    for name, o in seq:
        run(name, table, idx_dev, out, z.LaunchOpts(**o), idx.size, cfg.row_bytes)
    table.close()
    n_rows, n_idx = 4_000_000, 400_000
    idx_dev = torch.from_numpy(wl.uniform_indices(n_idx, n_rows, seed=5)).cuda()
    for dim in (128, 64, 32, 16):
        rb = dim * 4
        base = z.alloc_table(n_rows + 2, dim, "f32")
        out = torch.empty((n_idx, dim), dtype=torch.float32, device="cuda")
        wide = rb > 128
        for off in ((0, 128) if rb >= 128 else (0,)):
            view = z.table_view(base, off, n_rows, dim, "f32")  # stays host-resident
            o = z.LaunchOpts(variant=z.VARIANT_ROWVEC, unroll=2, max_blocks=2048 if wide else 8192,
                             vec_bytes=8 if wide else 16, group_lanes=64 if wide else 16)
            run(f"rows {rb} B base+{off}", view, idx_dev, out, o, n_idx, rb)
            if off == 0 and rb in (128, 256):
                for b in (8, 16, 32, 64, 128, 256):
                    o = z.LaunchOpts(variant=z.VARIANT_ROWVEC, unroll=2, max_blocks=b,
                                     vec_bytes=8 if wide else 16, group_lanes=64)
                    run(f"rows {rb} B base+0 {b} blocks", view, idx_dev, out, o, n_idx, rb)
            view.close()
        if rb == 64:  # the same rows through one 64-byte scalar read each
            run("rows 64 B base+0 scalar reads", base, idx_dev, out, z.LaunchOpts(variant=z.VARIANT_HALFLINE), n_idx, rb)
        base.close()
    return labels


def run_list_length(args, z, wl, np, torch, link_peak):
    """Gather time against list length for rows of 512 B ... 1 MiB: where the launch and the first
    round trip dominate, where the link fills, and what giving several wavefronts to one long
    row (row_splits) is worth on short lists of long rows."""
    cur = torch.cuda.current_stream()

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        ms = []
        for _ in range(max(10, min(args.steps, 30))):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(cur)
            fn()
            e1.record(cur)
            e1.synchronize()
            ms.append(e0.elapsed_time(e1))
        return float(np.median(ms))

    pts = []
    for dim, n_rows in ((128, 2_000_000), (1024, 500_000), (16_384, 40_000), (262_144, 2_000)):
        table = z.alloc_table(n_rows, dim, "f32")
        wl.fill_table_ptr(table.host_ptr, n_rows, dim, "f32", seed=wl.MASTER_SEED + 9)
        rb = dim * 4
        for n_idx in (1, 4, 16, 64, 256, 1024, 4096, 16384, 65536):
            if n_idx * rb > 1.2e9:
                break
            idx = torch.from_numpy(wl.uniform_indices(n_idx, n_rows, seed=n_idx)).cuda()
            out = torch.empty((n_idx, dim), dtype=torch.float32, device="cuda")
            plan = z.plan_gather(table, n_idx, out)
            us = timed(lambda: z.gather(table, idx, out, stream=cur)) * 1e3
            pt = {"row_bytes": rb, "n_idx": n_idx, "us": round(us, 1),
                  "gbps": round(n_idx * rb / us / 1e3, 2), "row_splits": plan["row_splits"]}
            if plan["row_splits"] > 1:
                one = z.LaunchOpts(row_splits=1)
                us1 = timed(lambda: z.gather_ex(table, idx, out, one, stream=cur)) * 1e3
                pt["us_one_wavefront_per_row"] = round(us1, 1)
            pts.append(pt)
            print(f"# {pt}", file=sys.stderr, flush=True)
        table.close()
    return pts


def run_table_size(args, z, wl, np, torch):
    """Does the link's request limit depend on how much memory the table spans? 1,000,000 uniform
    random rows of 128 bytes (one read request each) and of 512 bytes (bound by bytes) out of mapped
    tables of 0.13 ... 51 GB. The tables are left as allocated: only the rate matters here."""
    cur = torch.cuda.current_stream()
    n_idx = 1_000_000
    pts = []
    for dim, sizes in ((32, (1_000_000, 10_000_000, 100_000_000, 400_000_000)), (128, (10_000_000, 100_000_000))):
        for n_rows in sizes:
            if n_rows * dim * 4 > args.max_table_gb * 1e9:
                continue
            table = z.alloc_table(n_rows, dim, "f32")
            lists = [torch.from_numpy(wl.uniform_indices(n_idx, n_rows, seed=b)).cuda() for b in range(4)]
            out = torch.empty((n_idx, dim), dtype=torch.float32, device="cuda")
            for i in range(3):
                z.gather(table, lists[i % 4], out, stream=cur)
            torch.cuda.synchronize()
            ms = []
            for i in range(max(12, min(args.steps, 40))):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(cur)
                z.gather(table, lists[i % 4], out, stream=cur)
                e1.record(cur)
                e1.synchronize()
                ms.append(e0.elapsed_time(e1))
            m = float(np.median(ms))
            pt = {"row_bytes": dim * 4, "table_gb": round(n_rows * dim * 4 / 1e9, 2),
                  "rows_per_s_M": round(n_idx / m / 1e3, 1), "gbps": round(n_idx * dim * 4 / m / 1e6, 2)}
            pts.append(pt)
            print(f"# {pt}", file=sys.stderr, flush=True)
            table.close()
    return pts


def run_hbm_variant(args, z, wl, np, torch):
    """The all-in-GPU comparison variant (Section 4.1.2) against its own roofline: the same gather
    kernels on a table in HBM, with outputs far larger than the last-level cache, beside a plain
    device-to-device copy kernel of known size (what this chip's HBM sustains for read + write) and
    the framework's own row indexing."""
    cur = torch.cuda.current_stream()

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        ms = []
        for _ in range(max(10, min(args.steps, 30))):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(cur)
            fn()
            e1.record(cur)
            e1.synchronize()
            ms.append(e0.elapsed_time(e1))
        return float(np.median(ms))

    copies = []
    for gib in (0.5, 2, 8):
        n = int(gib * (1 << 30))
        a = torch.empty(n, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        ms = timed(lambda: probe.device_copy(b, a, n, cur))
        copies.append({"GiB": gib, "copy_gbps": round(n / ms / 1e6, 1), "traffic_TBps": round(2 * n / ms / 1e9, 2)})
        print(f"# {copies[-1]}", file=sys.stderr, flush=True)
        del a, b
    pts = []
    for dim, n_rows, n_idx in ((8, 10_000_000, 4_000_000), (32, 10_000_000, 4_000_000), (100, 10_000_000, 4_000_000),
                               (128, 10_000_000, 4_000_000), (602, 2_000_000, 1_000_000),
                               (1024, 2_500_000, 1_000_000)):
        src = torch.empty((n_rows, dim), dtype=torch.float32, device="cuda").uniform_(-1, 1)
        table = z.table_from_device(src.data_ptr(), n_rows, dim, "f32")
        idx = torch.from_numpy(wl.uniform_indices(n_idx, n_rows, seed=dim)).cuda()
        out = torch.empty((n_idx, dim), dtype=torch.float32, device="cuda")
        rb = dim * 4
        ms = timed(lambda: z.gather(table, idx, out, stream=cur))
        ms_lib = timed(lambda: torch.index_select(src, 0, idx, out=out))
        pt = {"row_bytes": rb, "out_MB": round(n_idx * rb / 1e6), "gathered_gbps": round(n_idx * rb / ms / 1e6, 1),
              "algorithmic_traffic_TBps": round(n_idx * (2 * rb + 8) / ms / 1e9, 2),
              "frac_of_8TBps": round(n_idx * (2 * rb + 8) / ms / 1e9 / 8.0, 3),
              "torch_index_select_gbps": round(n_idx * rb / ms_lib / 1e6, 1)}
        pts.append(pt)
        print(f"# {pt}", file=sys.stderr, flush=True)
        table.close()
        del src, out
    return {"plain_copy_kernel": copies, "gather": pts}
