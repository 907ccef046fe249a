"""GPU parity at the full sizes of the five workloads, in the launch
configuration the benchmark times (default options of zcg_gather): every output
byte against the CPU oracle, plus the closed-form table value recomputed here
for sampled elements (so the check does not rest on the oracle alone)."""
import numpy as np
import pytest

import zcg_workload as wl
from oracle import gather_bytes

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
z = pytest.importorskip("paper_2103_03330_amd")

U64 = np.uint64


def closed_form(seed, pos, dtype):
    """table[r, c] as a function of (seed, r*dim + c); independent restatement of the fill rule."""
    with np.errstate(over="ignore"):
        zz = U64(seed) + (pos.astype(U64) + U64(1)) * U64(0x9E3779B97F4A7C15)
        zz = (zz ^ (zz >> U64(30))) * U64(0xBF58476D1CE4E5B9)
        zz = (zz ^ (zz >> U64(27))) * U64(0x94D049BB133111EB)
        zz = zz ^ (zz >> U64(31))
    if dtype == "f32":
        return (((zz >> U64(40)).astype(np.int64) - (1 << 23)).astype(np.float64) * 2.0 ** -23).astype(np.float32)
    return (((zz >> U64(53)).astype(np.int64) - 1024).astype(np.float64) * 2.0 ** -10).astype(np.float16)


def check_config(cfg, lists, n_rows=None, also_hbm=False, full_oracle_on=None):
    n_rows = n_rows or cfg.n_rows
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    torch.cuda.set_device(0)
    print(f"[{cfg.name}] table {n_rows} x {cfg.dim} {cfg.dtype} ({n_rows * cfg.row_bytes / 1e9:.2f} GB), "
          f"{len(lists)} lists", flush=True)
    table = z.alloc_table(n_rows, cfg.dim, cfg.dtype)
    try:
        wl.fill_table_ptr(table.host_ptr, n_rows, cfg.dim, cfg.dtype, cfg.seed)
        tdt = torch.float32 if cfg.dtype == "f32" else torch.float16
        ndt = np.float32 if cfg.dtype == "f32" else np.float16
        rng = np.random.default_rng(7)
        hbm = None
        if also_hbm:
            hbm_t = torch.empty((n_rows, cfg.dim), dtype=tdt, device="cuda")
            step = max(1, (1 << 30) // cfg.row_bytes)
            host = table.host_array()
            for lo in range(0, n_rows, step):
                hbm_t[lo:lo + step].copy_(torch.from_numpy(host[lo:lo + step]))
            hbm = z.table_from_device(hbm_t, n_rows, cfg.dim, cfg.dtype)
        for b, idx in enumerate(lists):
            assert idx.min() >= 0 and idx.max() < n_rows
            idx_dev = torch.from_numpy(idx).cuda()
            assert z.validate_indices(table, idx_dev) == 0
            full = full_oracle_on is None or b in full_oracle_on
            if full:
                want = np.empty((idx.size, cfg.dim), dtype=ndt)
                gather_bytes(table.host_ptr, n_rows, cfg.row_bytes, idx, want.ctypes.data, n_threads=8)
            for t in ([table, hbm] if hbm else [table]):
                out = torch.zeros((idx.size, cfg.dim), dtype=tdt, device="cuda")
                z.gather(t, idx_dev, out)
                torch.cuda.synchronize()
                got = out.cpu().numpy()
                if full:
                    assert got.tobytes() == want.tobytes(), f"{cfg.name} list {b}: GPU differs from oracle"
            # sampled elements against the closed form
            n_samples = 4096 if full else 16384
            rows = rng.integers(0, idx.size, n_samples)
            cols = rng.integers(0, cfg.dim, n_samples)
            pos = idx[rows] * cfg.dim + cols
            assert (got[rows, cols] == closed_form(cfg.seed, pos, cfg.dtype)).all()
        if hbm:
            hbm.close()
    finally:
        table.close()


@pytest.mark.parametrize("k", [1, 2, 3])
def test_configs_1_to_3_full_size(k):
    cfg = wl.config(k)
    lists = wl.index_lists(cfg)
    if k == 3:  # secondary order: ascending
        lists = lists + [np.sort(lists[0])]
    check_config(cfg, lists, also_hbm=True)


def test_config_4_beyond_hbm_scale():
    """111 M x 128 fp32 = 56.8 GB of pinned host memory, the 50 minibatches the benchmark runs:
    three are compared byte for byte with the oracle, all 50 on 16,384 sampled elements each
    against the closed form of the table."""
    cfg = wl.config(4)
    g = wl.PowerLawGraph(cfg.n_rows, cfg.graph[0], cfg.graph[1], cfg.seed)
    lists = [g.sample_minibatch(cfg.n_seeds, cfg.fanout, b)[0] for b in range(50)]
    g.close()
    assert max(int(a.max()) for a in lists) * cfg.row_bytes > 2 ** 35  # offsets far beyond 32 bits
    check_config(cfg, lists, full_oracle_on=(0, 1, 49))


@pytest.mark.parametrize("cfg", wl.sweep_configs(), ids=lambda c: c.name)
def test_config_5_width_dtype_sweep(cfg):
    lists = wl.index_lists(cfg)
    check_config(cfg, lists, also_hbm=cfg.table_bytes <= 12e9)
