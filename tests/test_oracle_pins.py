"""Pins of the CPU oracle against things other than itself (no GPU needed).

The gather has an exact definition, out[i, c] = table[idx[i], c] (Section 3.2.1,
Listing 2), so the pins are: a pure-Python triple loop on tiny inputs,
invariants that only the correct gather satisfies, a table whose every element
is a closed-form function of its position (re-derived here in numpy, not taken
from the generator), numpy.take as an outside opinion, and planted mistakes
that the pins must catch.
"""
import numpy as np
import pytest

import zcg_workload as wl
from oracle import gather as oracle_gather, gather_bytes, OracleRangeError

U64 = np.uint64
GOLD = U64(0x9E3779B97F4A7C15)


def _mix64(z):
    z = (z ^ (z >> U64(30))) * U64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> U64(27))) * U64(0x94D049BB133111EB)
    return z ^ (z >> U64(31))


def closed_form(seed, pos, dtype):
    """Independent numpy statement of the table-fill rule: element at flat
    position p is a function of (seed, p) only."""
    with np.errstate(over="ignore"):
        z = _mix64(U64(seed) + (pos.astype(U64) + U64(1)) * GOLD)
    if dtype == "f32":
        k = (z >> U64(40)).astype(np.int64)
        return ((k - (1 << 23)).astype(np.float64) * 2.0 ** -23).astype(np.float32)
    k = (z >> U64(53)).astype(np.int64)
    return ((k - 1024).astype(np.float64) * 2.0 ** -10).astype(np.float16)


def brute_force(table, idx):
    out = np.zeros((len(idx), table.shape[1]), dtype=table.dtype)
    for i in range(len(idx)):
        for c in range(table.shape[1]):
            out[i, c] = table[idx[i], c]
    return out


def same_bits(a, b):
    return a.shape == b.shape and a.dtype == b.dtype and a.tobytes() == b.tobytes()


@pytest.mark.parametrize("n_rows,dim,dtype", [(7, 3, "f32"), (5, 1, "f32"), (1, 1, "f16"),
                                              (9, 5, "f16"), (13, 100, "f32"), (4, 602, "f32"),
                                              (11, 7, "f16")])
@pytest.mark.parametrize("n_idx", [0, 1, 17])
def test_brute_force_tiny(n_rows, dim, dtype, n_idx):
    table = wl.make_table(n_rows, dim, dtype, seed=11 + n_rows)
    idx = wl.uniform_indices(n_idx, n_rows, seed=dim)
    got = oracle_gather(table, idx)
    assert same_bits(got, brute_force(table, idx))


def test_raw_bit_patterns_are_moved_untouched():
    table = wl.make_table(64, 33, "f32", seed=5, mode=wl.FILL_RAW_BITS)
    bits = table.view(np.uint32)
    assert np.isnan(table).any()  # the fill really contains NaN payloads
    idx = wl.uniform_indices(200, 64, seed=9)
    got = oracle_gather(table, idx)
    assert same_bits(got.view(np.uint32), brute_force(bits, idx))
    t16 = wl.make_table(64, 33, "f16", seed=5, mode=wl.FILL_RAW_BITS)
    got16 = oracle_gather(t16, idx)
    assert same_bits(got16.view(np.uint16), brute_force(t16.view(np.uint16), idx))


@pytest.mark.parametrize("dtype,dim", [("f32", 100), ("f16", 37), ("f32", 128)])
def test_invariants(dtype, dim):
    n_rows = 301
    table = wl.make_table(n_rows, dim, dtype, seed=77)
    rng = np.random.default_rng(3)
    # identity list reproduces the table
    assert same_bits(oracle_gather(table, np.arange(n_rows)), table)
    # duplicates give identical rows
    idx = np.array([5, 9, 5, 5, 300, 9, 0], dtype=np.int64)
    out = oracle_gather(table, idx)
    assert same_bits(out[0], out[2]) and same_bits(out[2], out[3]) and same_bits(out[1], out[5])
    assert not same_bits(out[0], out[1])
    # permuting the list permutes the rows
    idx = rng.integers(0, n_rows, 500)
    perm = rng.permutation(500)
    assert same_bits(oracle_gather(table, idx[perm]), oracle_gather(table, idx)[perm])
    # composition and concatenation
    a = rng.integers(0, n_rows, 120)
    b = rng.integers(0, 120, 64)
    assert same_bits(oracle_gather(oracle_gather(table, a), b), oracle_gather(table, a[b]))
    assert same_bits(oracle_gather(table, np.concatenate([a, idx])),
                     np.concatenate([oracle_gather(table, a), oracle_gather(table, idx)]))


@pytest.mark.parametrize("dtype,n_rows,dim", [("f32", 5000, 100), ("f16", 3000, 257),
                                              ("f32", 1000, 602)])
def test_closed_form_table(dtype, n_rows, dim):
    seed = 210303330
    table = wl.make_table(n_rows, dim, dtype, seed)
    idx = wl.uniform_indices(4096, n_rows, seed=4)
    out = oracle_gather(table, idx, n_threads=3)
    pos = idx[:, None] * dim + np.arange(dim)[None, :]
    assert same_bits(out, closed_form(seed, pos, dtype))
    # the fill itself: uniform on [-1, 1), all values exactly on the stated grid
    assert out.min() >= -1 and out.max() < 1
    assert abs(float(out.astype(np.float64).mean())) < 0.02


def test_numpy_take_agrees_and_threads_do_not_matter():
    table = wl.make_table(20000, 100, "f32", seed=1)
    idx = wl.uniform_indices(70001, 20000, seed=2)
    ref = np.take(table, idx, axis=0)
    for nt in (1, 2, 8):
        assert same_bits(oracle_gather(table, idx, n_threads=nt), ref)


def test_out_of_range_is_an_error_and_leaves_output_alone():
    table = wl.make_table(10, 4, "f32", seed=1)
    out = np.full((3, 4), 7.0, dtype=np.float32)
    for bad in (10, -1, 2 ** 40):
        idx = np.array([1, bad, 2], dtype=np.int64)
        with pytest.raises(OracleRangeError, match="position 1"):
            gather_bytes(table.ctypes.data, 10, 16, idx, out.ctypes.data)
        assert (out == 7.0).all()
    with pytest.raises(ValueError):
        gather_bytes(table.ctypes.data, 10, 0, np.array([0]), out.ctypes.data)


def test_offsets_are_64_bit():
    # idx * row_bytes beyond 2^32 without a huge allocation: a wide virtual table
    # backed by one sparse mapping; only the rows named are touched.
    n_rows, row_bytes = 3_000_000, 2408
    table = np.lib.format.open_memmap("/tmp/_zcg_sparse_table.npy", mode="w+", dtype=np.uint8,
                                      shape=(n_rows, row_bytes))
    try:
        rows = np.array([0, n_rows - 1, 1_900_000, 2_000_123], dtype=np.int64)
        assert int(rows[-1]) * row_bytes > 2 ** 32
        for r in rows:
            table[r] = (np.arange(row_bytes) * 7 + r) % 251
        out = oracle_gather(table, rows)
        for i, r in enumerate(rows):
            assert (out[i] == (np.arange(row_bytes) * 7 + r) % 251).all()
    finally:
        del table
        import os
        os.unlink("/tmp/_zcg_sparse_table.npy")


# ---- planted mistakes: each plausible bug must trip at least one pin above ----

def _check_all_pins(g):
    """Runs a reduced set of the pins on gather function g; True if all pass."""
    table = wl.make_table(301, 100, "f32", seed=77)
    rng = np.random.default_rng(3)
    idx = rng.integers(0, 301, 500)
    perm = rng.permutation(500)
    ok = same_bits(g(table, np.arange(301)), table)
    ok &= same_bits(g(table, idx), brute_force(table, idx))
    ok &= same_bits(g(table, idx[perm]), g(table, idx)[perm])
    pos = idx[:, None] * 100 + np.arange(100)[None, :]
    ok &= same_bits(g(table, idx), closed_form(77, pos, "f32"))
    return bool(ok)


def test_planted_mistakes_are_caught():
    assert _check_all_pins(lambda t, i: oracle_gather(t, i))
    wrong = {
        "reversed list": lambda t, i: oracle_gather(t, i[::-1]),
        "off by one row": lambda t, i: oracle_gather(t, np.minimum(i + 1, t.shape[0] - 1)),
        "transposed operand": lambda t, i: oracle_gather(
            np.ascontiguousarray(t.T[: t.shape[1], : t.shape[1]]), i % t.shape[1]),
        "rotated row": lambda t, i: np.roll(oracle_gather(t, i), 1, axis=1),
        "dropped tail element": lambda t, i: np.concatenate(
            [oracle_gather(t, i)[:, :-1], np.zeros((len(i), 1), t.dtype)], axis=1),
        "sorted list": lambda t, i: oracle_gather(t, np.sort(i)),
    }
    for name, g in wrong.items():
        assert not _check_all_pins(g), f"planted mistake not caught: {name}"
