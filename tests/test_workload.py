"""Host-side checks of the synthetic input generators (no GPU needed)."""
import numpy as np
import pytest

import zcg_workload as wl


def test_fill_is_position_keyed_and_thread_independent():
    a = wl.make_table(1000, 37, "f32", seed=9, n_threads=1)
    b = wl.make_table(1000, 37, "f32", seed=9, n_threads=5)
    assert a.tobytes() == b.tobytes()
    # a taller table with the same width starts with the same rows
    c = wl.make_table(1500, 37, "f32", seed=9)
    assert c[:1000].tobytes() == a.tobytes()
    assert wl.make_table(1000, 37, "f32", seed=10).tobytes() != a.tobytes()


def test_fp16_values_are_exact_grid_points():
    t = wl.make_table(4096, 8, "f16", seed=3).astype(np.float64)
    k = t * 1024 + 1024
    assert (k == np.round(k)).all() and k.min() >= 0 and k.max() <= 2047
    assert len(np.unique(k)) > 1500


def test_uniform_indices_distribution():
    idx = wl.uniform_indices(65536, 100000, seed=1)
    assert idx.min() >= 0 and idx.max() < 100000
    distinct = len(np.unique(idx))
    # 65,536 draws from 100,000: expected distinct = n(1 - exp(-m/n)) ~ 48,070
    assert 47000 < distinct < 49000


@pytest.fixture(scope="module")
def small_graph():
    g = wl.PowerLawGraph(200_000, 50.0, 2.1, seed=42)
    yield g
    g.close()


def test_graph_mean_degree_and_hubs(small_graph):
    g = small_graph
    deg = np.array([g.degree(u) for u in range(0, g.n, 7)])
    assert abs(deg.mean() - 50.0) / 50.0 < 0.03
    assert deg.min() >= 1
    assert deg.max() <= np.sqrt(g.n * 50.0) * 1.01
    # heavy tail: the top 1% of nodes hold well over 10% of the degree mass
    top = np.sort(deg)[-len(deg) // 100:]
    assert top.sum() / deg.sum() > 0.10


def test_label_permutation_is_a_bijection():
    g = wl.PowerLawGraph(1009, 10.0, 2.1, seed=5)
    p = g.params()
    labels = {(p["A"] * j + p["B"]) % g.n for j in range(g.n)}
    assert len(labels) == g.n
    assert (p["A"] * p["Ainv"]) % g.n == 1
    g.close()


def test_neighbors_are_fixed_valid_and_weight_proportional(small_graph):
    g = small_graph
    for u in (0, 17, g.n - 1):
        nb = [g.neighbor(u, p) for p in range(g.degree(u))]
        assert nb == [g.neighbor(u, p) for p in range(g.degree(u))]
        assert all(0 <= v < g.n and v != u for v in nb)
    # nodes are named as neighbors in proportion to their expected degree
    draws = np.array([g.neighbor(u, p) for u in range(0, 20000) for p in range(5)])
    counts = np.bincount(draws, minlength=g.n)
    hubs = np.argsort(counts)[-50:]
    hub_deg = np.array([g.degree(int(u)) for u in hubs])
    assert hub_deg.mean() > 20 * 50.0


def test_minibatch_structure(small_graph):
    g = small_graph
    idx, hop_end = g.sample_minibatch(256, (15, 10), batch_id=3)
    assert len(idx) == hop_end[-1] and hop_end[0] == 256
    assert len(np.unique(idx)) == len(idx)  # deduplicated
    assert idx.min() >= 0 and idx.max() < g.n
    assert hop_end[1] <= 256 * 16 and hop_end[2] <= 256 * 16 * 11
    # hop-1 nodes are neighbors of seeds
    seeds = idx[:256]
    seed_nb = set()
    for u in seeds:
        seed_nb.update(g.neighbor(int(u), p) for p in range(g.degree(int(u))))
    assert set(idx[256:hop_end[1]].tolist()) <= seed_nb
    # hop-2 nodes are neighbors of some node found before hop 2
    prior_nb = set()
    for u in idx[:hop_end[1]]:
        prior_nb.update(g.neighbor(int(u), p) for p in range(g.degree(int(u))))
    assert set(idx[hop_end[1]:].tolist()) <= prior_nb
    # deterministic per batch id, different across batch ids
    again, _ = g.sample_minibatch(256, (15, 10), batch_id=3)
    other, _ = g.sample_minibatch(256, (15, 10), batch_id=4)
    assert (again == idx).all() and not np.array_equal(other, idx)


def test_fanout_is_without_replacement_on_positions():
    g = wl.PowerLawGraph(5000, 40.0, 2.1, seed=8)
    idx, hop_end = g.sample_minibatch(1, (10,), batch_id=0)
    u = int(idx[0])
    got = idx[1:]
    assert len(got) <= min(10, g.degree(u))
    # a low-degree node contributes its whole list
    low = min(range(g.n), key=g.degree)
    assert g.degree(low) < 64
    g.close()


def test_config_shapes():
    c2, c3, c4 = wl.config(2), wl.config(3), wl.config(4)
    assert c2.row_bytes == 400 and c3.row_bytes == 2408 and c4.row_bytes == 512
    assert c4.table_bytes == 111_000_000 * 512
    assert len(wl.sweep_configs()) == 8
    assert {c.row_bytes for c in wl.sweep_configs()} == {32, 128, 512, 2048, 64, 256, 1024, 4096}
    lists = wl.index_lists(wl.config(1))
    assert len(lists) == 1 and len(lists[0]) == 65536
