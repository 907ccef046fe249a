"""Seeded synthetic inputs for the zero-copy feature gather.

This package only *produces inputs*: feature tables, uniform index lists and
k-hop neighbor-sampled node-ID lists (the sampler -> producer hand-off of the
paper's Section 3.3). It performs no gather and is shared by the CPU oracle
tests and the GPU path; neither of those imports the other.

The generators are native (C + OpenMP, ``csrc/workload.c``) because the largest
table is tens of GB; ``build()`` compiles them with gcc.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csrc", "workload.c")
_LIB_PATH = os.path.join(_HERE, "libzcg_workload.so")

MASTER_SEED = 210303330

FILL_UNIFORM = 0  # exactly representable values on [-1, 1)
FILL_RAW_BITS = 1  # arbitrary bit patterns (NaN payloads, -0.0, denormals)


def build(verbose: bool = False) -> str:
    """Compile the generator library in-tree with gcc."""
    cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=gnu11", "-o", _LIB_PATH, _SRC, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    global _lib
    _lib = None
    return _LIB_PATH


_lib = None


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        build()
    lib = ctypes.CDLL(_LIB_PATH)
    i64, u64, i32, vp, dbl = (ctypes.c_int64, ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p,
                              ctypes.c_double)
    lib.zcgw_fill_table.argtypes = [vp, i64, i64, i32, u64, i32, i32]
    lib.zcgw_fill_table.restype = i32
    lib.zcgw_uniform_indices.argtypes = [vp, i64, i64, u64, i32]
    lib.zcgw_uniform_indices.restype = i32
    lib.zcgw_graph_create.argtypes = [i64, dbl, dbl, u64]
    lib.zcgw_graph_create.restype = vp
    lib.zcgw_graph_destroy.argtypes = [vp]
    lib.zcgw_graph_destroy.restype = None
    lib.zcgw_graph_degree.argtypes = [vp, i64]
    lib.zcgw_graph_degree.restype = i64
    lib.zcgw_graph_neighbor.argtypes = [vp, i64, i64]
    lib.zcgw_graph_neighbor.restype = i64
    lib.zcgw_graph_params.argtypes = [vp, vp]
    lib.zcgw_graph_params.restype = None
    lib.zcgw_sample_minibatch.argtypes = [vp, i64, vp, i32, u64, vp, i64, vp]
    lib.zcgw_sample_minibatch.restype = i64
    _lib = lib
    return lib


def default_threads() -> int:
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        return int(env)
    try:
        return max(1, len(os.sched_getaffinity(0)))
    except AttributeError:
        return max(1, os.cpu_count() or 1)


_ELEM = {"f16": 2, "f32": 4, "i8": 1, "f64": 8}
_NP = {"f16": np.float16, "f32": np.float32, "i8": np.int8, "f64": np.float64}


def elem_bytes(dtype: str) -> int:
    return _ELEM[dtype]


def fill_table_ptr(ptr: int, n_rows: int, dim: int, dtype: str, seed: int,
                   mode: int = FILL_UNIFORM, n_threads: Optional[int] = None) -> None:
    """Fill caller-owned memory at address ``ptr`` (e.g. pinned host memory)."""
    rc = _load().zcgw_fill_table(ctypes.c_void_p(ptr), n_rows, dim, _ELEM[dtype],
                                 seed & (2**64 - 1), mode, n_threads or default_threads())
    if rc != 0:
        raise ValueError("zcgw_fill_table: bad arguments")


def make_table(n_rows: int, dim: int, dtype: str, seed: int, mode: int = FILL_UNIFORM,
               n_threads: Optional[int] = None) -> np.ndarray:
    """A new pageable numpy table [n_rows, dim] of the given dtype."""
    t = np.empty((n_rows, dim), dtype=_NP[dtype])
    if t.size:
        fill_table_ptr(t.ctypes.data, n_rows, dim, dtype, seed, mode, n_threads)
    return t


def uniform_indices(n_idx: int, n_rows: int, seed: int, n_threads: Optional[int] = None) -> np.ndarray:
    idx = np.empty(n_idx, dtype=np.int64)
    rc = _load().zcgw_uniform_indices(ctypes.c_void_p(idx.ctypes.data), n_idx, n_rows,
                                      seed & (2**64 - 1), n_threads or default_threads())
    if rc != 0:
        raise ValueError("zcgw_uniform_indices: bad arguments")
    return idx


class PowerLawGraph:
    """Implicit Chung-Lu style power-law graph (see csrc/workload.c for the recipe)."""

    def __init__(self, n: int, avg_deg: float, gamma: float, seed: int):
        self._lib = _load()
        self.n, self.avg_deg, self.gamma, self.seed = n, avg_deg, gamma, seed
        self._h = self._lib.zcgw_graph_create(n, float(avg_deg), float(gamma), seed & (2**64 - 1))
        if not self._h:
            raise ValueError("zcgw_graph_create: bad arguments or out of memory")

    def close(self) -> None:
        if getattr(self, "_h", None):
            self._lib.zcgw_graph_destroy(self._h)
            self._h = None

    __del__ = close

    def degree(self, u: int) -> int:
        return int(self._lib.zcgw_graph_degree(self._h, u))

    def neighbor(self, u: int, pos: int) -> int:
        return int(self._lib.zcgw_graph_neighbor(self._h, u, pos))

    def params(self) -> dict:
        buf = (ctypes.c_double * 6)()
        self._lib.zcgw_graph_params(self._h, buf)
        return dict(j0=buf[0], c=buf[1], a=buf[2], A=int(buf[3]), B=int(buf[4]), Ainv=int(buf[5]))

    def sample_minibatch(self, n_seeds: int, fanout: Sequence[int], batch_id: int = 0
                         ) -> Tuple[np.ndarray, List[int]]:
        """Deduplicated node-ID list in first-occurrence order and the list
        length after the seeds and after each hop."""
        cap = n_seeds
        for f in fanout:
            cap = min(self.n, cap * (f + 1))
        out = np.empty(cap, dtype=np.int64)
        fo = np.asarray(fanout, dtype=np.int32)
        hop_end = np.zeros(len(fanout) + 1, dtype=np.int64)
        n = self._lib.zcgw_sample_minibatch(self._h, n_seeds, ctypes.c_void_p(fo.ctypes.data),
                                            len(fo), batch_id & (2**64 - 1),
                                            ctypes.c_void_p(out.ctypes.data), cap,
                                            ctypes.c_void_p(hop_end.ctypes.data))
        if n < 0:
            raise ValueError(f"zcgw_sample_minibatch failed ({n})")
        return out[:n].copy(), [int(x) for x in hop_end]


@dataclass(frozen=True)
class GatherConfig:
    """Shape of one synthetic workload. ``graph`` is None for uniform index lists."""
    name: str
    n_rows: int
    dim: int
    dtype: str
    n_idx: int = 0  # uniform lists only
    graph: Optional[Tuple[float, float]] = None  # (avg_deg, gamma)
    n_seeds: int = 0
    fanout: Tuple[int, ...] = ()
    n_batches: int = 1
    seed: int = MASTER_SEED

    @property
    def row_bytes(self) -> int:
        return self.dim * _ELEM[self.dtype]

    @property
    def table_bytes(self) -> int:
        return self.n_rows * self.row_bytes


def config(k: int) -> GatherConfig:
    """Configs 1-4 as listed for this build (config 5 is ``sweep_configs``)."""
    s = MASTER_SEED + k
    if k == 1:
        return GatherConfig("cfg1_tiny", 100_000, 128, "f32", n_idx=65_536, seed=s)
    if k == 2:
        return GatherConfig("cfg2_unaligned_400B", 2_450_000, 100, "f32", graph=(50.0, 2.1),
                            n_seeds=1024, fanout=(15, 10), seed=s)
    if k == 3:
        return GatherConfig("cfg3_wide_2408B", 233_000, 602, "f32", graph=(490.0, 2.1),
                            n_seeds=1000, fanout=(25, 10), seed=s)
    if k == 4:
        return GatherConfig("cfg4_scale_56GB", 111_000_000, 128, "f32", graph=(30.0, 2.1),
                            n_seeds=1024, fanout=(15, 10, 5), n_batches=50, seed=s)
    raise ValueError("config index must be 1..4")


def sweep_configs() -> List[GatherConfig]:
    """Config 5: 10M rows x dim in {16,64,256,1024}, fp16 and fp32, 1M uniform indices."""
    out = []
    for dtype in ("f16", "f32"):
        for dim in (16, 64, 256, 1024):
            out.append(GatherConfig(f"cfg5_{dtype}_d{dim}", 10_000_000, dim, dtype,
                                    n_idx=1_000_000, seed=MASTER_SEED + 5))
    return out


def index_lists(cfg: GatherConfig, n_rows: Optional[int] = None) -> List[np.ndarray]:
    """The int64 index list(s) of a config: one per minibatch. ``n_rows`` overrides
    the table height (used when a table had to be scaled down to fit host memory)."""
    n = n_rows or cfg.n_rows
    if cfg.graph is None:
        return [uniform_indices(cfg.n_idx, n, cfg.seed ^ 0x1D)]
    g = PowerLawGraph(n, cfg.graph[0], cfg.graph[1], cfg.seed)
    try:
        return [g.sample_minibatch(cfg.n_seeds, cfg.fanout, b)[0] for b in range(cfg.n_batches)]
    finally:
        g.close()
