"""ctypes binding of libzcgather: argument marshalling only.

Every function mirrors one C entry point of ``include/zcgather.h`` (same name
without the ``zcg_`` prefix). Pointers may be given as integers or as objects
with a ``data_ptr()`` method (torch tensors); streams as integers, objects with
a ``cuda_stream`` attribute (torch streams) or None for the default stream.
There is no CPU fallback: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import build as _build

# status codes / constants (include/zcgather.h)
OK, EINVAL, EDTYPE, EHANDLE, EHIP, ENOMEM, EALIGN, EALIAS, ERANGE, EBUSY, ETIMEDOUT, ECLOSED, ECAPACITY = (
    0, -1, -2, -3, -4, -5, -6, -7, -8, -9, -10, -11, -12)
F16, F32, B8, B64 = 1, 2, 3, 4
ALLOC_DEFAULT, ALLOC_NONCOHERENT, ALLOC_NUMA_USER, ALLOC_UNCACHED = 0, 1, 2, 4
VARIANT_AUTO, VARIANT_NAIVE, VARIANT_ROWVEC, VARIANT_ALIGNED, VARIANT_HALFLINE = 0, 1, 2, 3, 4
VARIANT_NAMES = {VARIANT_AUTO: "auto", VARIANT_NAIVE: "naive", VARIANT_ROWVEC: "rowvec",
                 VARIANT_ALIGNED: "aligned", VARIANT_HALFLINE: "halfline"}
_DTYPES = {"f16": F16, "f32": F32, "i8": B8, "f64": B64, F16: F16, F32: F32, B8: B8, B64: B64}
_ELEM = {F16: 2, F32: 4, B8: 1, B64: 8}
_NP = {F16: np.float16, F32: np.float32, B8: np.int8, B64: np.float64}

EXPORTS = [
    "zcg_strerror", "zcg_last_hip_error", "zcg_register_table", "zcg_alloc_table",
    "zcg_table_from_device", "zcg_table_device_ptr", "zcg_table_host_ptr", "zcg_table_row_bytes",
    "zcg_table_n_rows", "zcg_unregister_table", "zcg_gather", "zcg_gather_variant",
    "zcg_gather_ex", "zcg_plan_gather", "zcg_validate_indices", "zcg_cpu_gather_memcpy",
    "zcg_cpu_gather_memcpy_chunked", "zcg_pinned_alloc", "zcg_pinned_free",
    "zcg_version", "zcg_stream_create_cu_mask", "zcg_stream_destroy", "zcg_device_cu_count",
    "zcg_pipeline_create", "zcg_pipeline_submit", "zcg_pipeline_submit_wait",
    "zcg_pipeline_finish", "zcg_pipeline_next", "zcg_pipeline_acquire",
    "zcg_pipeline_release", "zcg_pipeline_destroy", "zcg_gather_ordered",
    "zcg_order_workspace_bytes", "zcg_make_order", "zcg_table_view", "zcg_gather_workspace_bytes",
    "zcg_make_order_static", "zcg_plan_shape",
]


class LaunchOpts(ctypes.Structure):
    """zcg_launch_opts; zero in a field means the library default."""
    _fields_ = [("variant", ctypes.c_int), ("max_blocks", ctypes.c_int), ("unroll", ctypes.c_int),
                ("line_bytes", ctypes.c_int), ("nt_loads", ctypes.c_int),
                ("nt_stores", ctypes.c_int), ("vec_bytes", ctypes.c_int),
                ("group_lanes", ctypes.c_int), ("shifted_stores", ctypes.c_int),
                ("row_splits", ctypes.c_int), ("half_ends", ctypes.c_int),
                ("workspace_dev", ctypes.c_void_p), ("workspace_bytes", ctypes.c_int64)]


class Plan(ctypes.Structure):
    """zcg_plan."""
    _fields_ = [("variant", ctypes.c_int), ("vec_bytes", ctypes.c_int),
                ("log2_group", ctypes.c_int), ("iters", ctypes.c_int), ("unroll", ctypes.c_int),
                ("line_bytes", ctypes.c_int), ("nt_loads", ctypes.c_int),
                ("nt_stores", ctypes.c_int), ("blocks", ctypes.c_int),
                ("store_bytes", ctypes.c_int), ("row_splits", ctypes.c_int),
                ("half_ends", ctypes.c_int), ("ordered", ctypes.c_int)]

    def as_dict(self) -> dict:
        return {k: getattr(self, k) for k, _ in self._fields_}


class ZcgError(RuntimeError):
    def __init__(self, status: int, what: str, hip_error: int = 0):
        self.status, self.hip_error = status, hip_error
        msg = f"{what}: {strerror(status)} ({status})"
        if status == EHIP:
            msg += f", hipError_t={hip_error}"
        super().__init__(msg)


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the built library; build it first only if nothing is built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB_PATH):
        _build.build()
    lib = ctypes.CDLL(_build.LIB_PATH)
    vp, i64, i32, u32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint
    pvp = ctypes.POINTER(ctypes.c_void_p)
    sigs = {
        "zcg_strerror": (ctypes.c_char_p, [i32]),
        "zcg_version": (ctypes.c_char_p, []),
        "zcg_last_hip_error": (i32, []),
        "zcg_register_table": (i32, [vp, i64, i64, i32, i32, pvp]),
        "zcg_alloc_table": (i32, [i64, i64, i32, u32, i32, pvp]),
        "zcg_table_from_device": (i32, [vp, i64, i64, i32, i32, pvp]),
        "zcg_table_device_ptr": (vp, [vp]),
        "zcg_table_host_ptr": (vp, [vp]),
        "zcg_table_row_bytes": (i64, [vp]),
        "zcg_table_n_rows": (i64, [vp]),
        "zcg_unregister_table": (i32, [vp]),
        "zcg_gather": (i32, [vp, vp, i64, vp, vp]),
        "zcg_gather_variant": (i32, [vp, vp, i64, vp, vp, i32]),
        "zcg_gather_ex": (i32, [vp, vp, i64, vp, vp, ctypes.POINTER(LaunchOpts)]),
        "zcg_plan_gather": (i32, [vp, i64, vp, ctypes.POINTER(LaunchOpts), ctypes.POINTER(Plan)]),
        "zcg_validate_indices": (i32, [vp, vp, i64, vp, ctypes.POINTER(i64)]),
        "zcg_cpu_gather_memcpy": (i32, [vp, vp, i64, vp, vp, i32, vp]),
        "zcg_cpu_gather_memcpy_chunked": (i32, [vp, vp, i64, vp, vp, i32, i64, vp]),
        "zcg_pinned_alloc": (i32, [i64, pvp]),
        "zcg_pinned_free": (i32, [vp]),
        "zcg_stream_create_cu_mask": (i32, [i32, ctypes.POINTER(ctypes.c_uint32), i32, pvp]),
        "zcg_stream_destroy": (i32, [vp]),
        "zcg_device_cu_count": (i32, [i32, ctypes.POINTER(i32)]),
        "zcg_pipeline_create": (i32, [vp, i64, i32, ctypes.POINTER(ctypes.c_void_p), vp, pvp]),
        "zcg_pipeline_submit": (i32, [vp, vp, i64, ctypes.POINTER(i32)]),
        "zcg_pipeline_submit_wait": (i32, [vp, vp, i64, i32, ctypes.POINTER(i32)]),
        "zcg_pipeline_finish": (i32, [vp]),
        "zcg_pipeline_next": (i32, [vp, i32, ctypes.POINTER(i32)]),
        "zcg_pipeline_acquire": (i32, [vp, i32, vp, pvp, ctypes.POINTER(i64)]),
        "zcg_pipeline_release": (i32, [vp, i32, vp]),
        "zcg_pipeline_destroy": (i32, [vp]),
        "zcg_gather_ordered": (i32, [vp, vp, vp, i64, vp, vp, ctypes.POINTER(LaunchOpts)]),
        "zcg_order_workspace_bytes": (i32, [i64, ctypes.POINTER(i64)]),
        "zcg_make_order": (i32, [vp, i64, i64, vp, vp, i64, vp]),
        "zcg_make_order_static": (i32, [vp, i64, i64, vp, vp]),
        "zcg_plan_shape": (i32, [i64, i32, ctypes.c_uint64, ctypes.c_uint64, i64, i64, i32,
                                 ctypes.POINTER(LaunchOpts), ctypes.POINTER(Plan)]),
        "zcg_table_view": (i32, [vp, i64, i64, i64, i32, pvp]),
        "zcg_gather_workspace_bytes": (i32, [i64, ctypes.POINTER(i64)]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load_library().zcg_strerror(status).decode()


def version() -> str:
    return load_library().zcg_version().decode()


def last_hip_error() -> int:
    return int(load_library().zcg_last_hip_error())


def _check(status: int, what: str) -> None:
    if status != OK:
        raise ZcgError(status, what, last_hip_error() if status == EHIP else 0)


def _ptr(x) -> int:
    if x is None:
        return 0
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    return int(x)


def _stream(s) -> int:
    if s is None:
        return 0
    if hasattr(s, "cuda_stream"):
        return int(s.cuda_stream)
    return int(s)


def _n_idx(idx, n_idx: Optional[int]) -> int:
    if n_idx is not None:
        return int(n_idx)
    if hasattr(idx, "numel"):
        return int(idx.numel())
    if hasattr(idx, "size"):
        return int(idx.size)
    raise TypeError("n_idx is required when idx is a raw pointer")


def _check_idx_tensor(idx) -> None:
    # torch tensors carry enough to catch the common marshalling mistakes early
    if hasattr(idx, "dtype") and hasattr(idx, "is_contiguous"):
        if "int64" not in str(idx.dtype):
            raise TypeError("index list must be int64")
        if not idx.is_contiguous():
            raise ValueError("index list must be contiguous")


@dataclass
class Table:
    """A live table handle. ``close()`` (or the context manager) unpins / frees it."""
    handle: int
    n_rows: int
    dim: int
    dtype: int

    @property
    def elem_bytes(self) -> int:
        return _ELEM[self.dtype]

    @property
    def row_bytes(self) -> int:
        return self.dim * self.elem_bytes

    @property
    def device_ptr(self) -> int:
        return int(load_library().zcg_table_device_ptr(self.handle) or 0)

    @property
    def host_ptr(self) -> int:
        return int(load_library().zcg_table_host_ptr(self.handle) or 0)

    def host_array(self) -> np.ndarray:
        """numpy view [n_rows, dim] of a host-resident table (no copy)."""
        p = self.host_ptr
        if not p:
            raise ValueError("table has no host address")
        n = self.n_rows * self.dim
        buf = (ctypes.c_char * (n * self.elem_bytes)).from_address(p)
        return np.frombuffer(buf, dtype=_NP[self.dtype], count=n).reshape(self.n_rows, self.dim)

    def close(self) -> None:
        if self.handle:
            h, self.handle = self.handle, 0
            _check(load_library().zcg_unregister_table(h), "zcg_unregister_table")

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def _new_table(status: int, what: str, out: ctypes.c_void_p, n_rows, dim, dtype) -> Table:
    _check(status, what)
    return Table(int(out.value), int(n_rows), int(dim), dtype)


def register_table(host, n_rows: int, dim: int, dtype, device: int = 0) -> Table:
    """Pin + map caller-owned host memory (a numpy array or an address)."""
    addr = host.ctypes.data if isinstance(host, np.ndarray) else _ptr(host)
    dt = _DTYPES.get(dtype, dtype)
    out = ctypes.c_void_p()
    rc = load_library().zcg_register_table(addr, n_rows, dim, dt, device, ctypes.byref(out))
    return _new_table(rc, "zcg_register_table", out, n_rows, dim, dt)


def alloc_table(n_rows: int, dim: int, dtype, flags: int = ALLOC_DEFAULT, device: int = 0) -> Table:
    dt = _DTYPES.get(dtype, dtype)
    out = ctypes.c_void_p()
    rc = load_library().zcg_alloc_table(n_rows, dim, dt, flags, device, ctypes.byref(out))
    return _new_table(rc, "zcg_alloc_table", out, n_rows, dim, dt)


def table_from_device(dev, n_rows: int, dim: int, dtype, device: int = 0) -> Table:
    dt = _DTYPES.get(dtype, dtype)
    out = ctypes.c_void_p()
    rc = load_library().zcg_table_from_device(_ptr(dev), n_rows, dim, dt, device, ctypes.byref(out))
    return _new_table(rc, "zcg_table_from_device", out, n_rows, dim, dt)


def table_view(parent: Table, byte_offset: int, n_rows: int, dim: int, dtype) -> Table:
    """A slice of a live table as a table of its own (no pinning, no copy)."""
    dt = _DTYPES.get(dtype, dtype)
    out = ctypes.c_void_p()
    rc = load_library().zcg_table_view(parent.handle, byte_offset, n_rows, dim, dt, ctypes.byref(out))
    return _new_table(rc, "zcg_table_view", out, n_rows, dim, dt)


def unregister_table(table: Table) -> None:
    table.close()


def gather(table: Table, idx_dev, out_dev, n_idx: Optional[int] = None, stream=None) -> None:
    _check_idx_tensor(idx_dev)
    rc = load_library().zcg_gather(table.handle, _ptr(idx_dev), _n_idx(idx_dev, n_idx),
                                   _ptr(out_dev), _stream(stream))
    _check(rc, "zcg_gather")


def gather_variant(table: Table, idx_dev, out_dev, variant: int, n_idx: Optional[int] = None,
                   stream=None) -> None:
    _check_idx_tensor(idx_dev)
    rc = load_library().zcg_gather_variant(table.handle, _ptr(idx_dev), _n_idx(idx_dev, n_idx),
                                           _ptr(out_dev), _stream(stream), variant)
    _check(rc, "zcg_gather_variant")


def gather_ex(table: Table, idx_dev, out_dev, opts: Optional[LaunchOpts] = None,
              n_idx: Optional[int] = None, stream=None) -> None:
    _check_idx_tensor(idx_dev)
    rc = load_library().zcg_gather_ex(table.handle, _ptr(idx_dev), _n_idx(idx_dev, n_idx),
                                      _ptr(out_dev), _stream(stream),
                                      ctypes.byref(opts) if opts is not None else None)
    _check(rc, "zcg_gather_ex")


def plan_gather(table: Table, n_idx: int, out_dev, opts: Optional[LaunchOpts] = None) -> dict:
    plan = Plan()
    rc = load_library().zcg_plan_gather(table.handle, n_idx, _ptr(out_dev),
                                        ctypes.byref(opts) if opts is not None else None,
                                        ctypes.byref(plan))
    _check(rc, "zcg_plan_gather")
    return plan.as_dict()


def plan_shape(row_bytes: int, elem_bytes: int, table_addr: int, out_addr: int, n_rows: int, n_idx: int,
               host_resident: bool, opts: Optional[LaunchOpts] = None) -> dict:
    """zcg_plan_shape: the launch plan for a table given by numbers (host-only)."""
    plan = Plan()
    rc = load_library().zcg_plan_shape(row_bytes, elem_bytes, table_addr, out_addr, n_rows, n_idx,
                                       1 if host_resident else 0,
                                       ctypes.byref(opts) if opts is not None else None, ctypes.byref(plan))
    _check(rc, "zcg_plan_shape")
    return plan.as_dict()


def validate_indices(table: Table, idx_dev, n_idx: Optional[int] = None, stream=None) -> int:
    _check_idx_tensor(idx_dev)
    n_bad = ctypes.c_int64(0)
    rc = load_library().zcg_validate_indices(table.handle, _ptr(idx_dev), _n_idx(idx_dev, n_idx),
                                             _stream(stream), ctypes.byref(n_bad))
    _check(rc, "zcg_validate_indices")
    return int(n_bad.value)


def _host_idx(idx_host) -> np.ndarray:
    a = np.ascontiguousarray(idx_host, dtype=np.int64)
    if a.ndim != 1:
        raise ValueError("index list must be 1-D")
    return a


def cpu_gather_memcpy(table: Table, idx_host, staging_pinned, out_dev, n_threads: int = 0,
                      stream=None) -> None:
    a = _host_idx(idx_host)
    rc = load_library().zcg_cpu_gather_memcpy(table.handle, a.ctypes.data, a.size,
                                              _ptr(staging_pinned), _ptr(out_dev), n_threads,
                                              _stream(stream))
    _check(rc, "zcg_cpu_gather_memcpy")


def cpu_gather_memcpy_chunked(table: Table, idx_host, staging_pinned, out_dev, chunk_rows: int,
                              n_threads: int = 0, stream=None) -> None:
    a = _host_idx(idx_host)
    rc = load_library().zcg_cpu_gather_memcpy_chunked(table.handle, a.ctypes.data, a.size,
                                                      _ptr(staging_pinned), _ptr(out_dev),
                                                      n_threads, chunk_rows, _stream(stream))
    _check(rc, "zcg_cpu_gather_memcpy_chunked")


def pinned_alloc(n_bytes: int) -> int:
    p = ctypes.c_void_p()
    _check(load_library().zcg_pinned_alloc(n_bytes, ctypes.byref(p)), "zcg_pinned_alloc")
    return int(p.value)


def pinned_free(ptr: int) -> None:
    _check(load_library().zcg_pinned_free(ptr), "zcg_pinned_free")


def device_cu_count(device: int = 0) -> int:
    n = ctypes.c_int(0)
    _check(load_library().zcg_device_cu_count(device, ctypes.byref(n)), "zcg_device_cu_count")
    return int(n.value)


class MaskedStream:
    """A HIP stream bound to a set of compute units (zcg_stream_create_cu_mask)."""

    def __init__(self, cu_ids, device: int = 0, n_words: int = 8):
        words = (ctypes.c_uint32 * n_words)()
        for c in cu_ids:
            if not 0 <= c < n_words * 32:
                raise ValueError("compute unit id out of range")
            words[c // 32] |= 1 << (c % 32)
        out = ctypes.c_void_p()
        _check(load_library().zcg_stream_create_cu_mask(device, words, n_words, ctypes.byref(out)),
               "zcg_stream_create_cu_mask")
        self.cuda_stream = int(out.value)
        self.cu_ids = list(cu_ids)

    def close(self) -> None:
        if self.cuda_stream:
            h, self.cuda_stream = self.cuda_stream, 0
            _check(load_library().zcg_stream_destroy(h), "zcg_stream_destroy")


def stream_create_cu_mask(cu_ids, device: int = 0) -> MaskedStream:
    return MaskedStream(cu_ids, device)


def stream_destroy(stream: MaskedStream) -> None:
    stream.close()


class Pipeline:
    """zcg_pipeline_*: ring of caller-owned output buffers fed by a gather stream."""

    def __init__(self, table: Table, max_rows: int, out_bufs, gather_stream=None):
        self._bufs = list(out_bufs)  # keep the tensors alive
        arr = (ctypes.c_void_p * len(self._bufs))(*[_ptr(b) for b in self._bufs])
        out = ctypes.c_void_p()
        _check(load_library().zcg_pipeline_create(table.handle, max_rows, len(self._bufs), arr,
                                                  _stream(gather_stream), ctypes.byref(out)),
               "zcg_pipeline_create")
        self.handle = int(out.value)

    def submit(self, idx_host, timeout_ms: Optional[int] = None) -> int:
        """Enqueue one minibatch; returns its slot. Without ``timeout_ms`` a ring that is full
        raises EBUSY at once; with it (negative = no limit) the call sleeps until the consumer
        thread releases the buffer."""
        a = _host_idx(idx_host)
        slot = ctypes.c_int(-1)
        if timeout_ms is None:
            _check(load_library().zcg_pipeline_submit(self.handle, a.ctypes.data, a.size,
                                                      ctypes.byref(slot)), "zcg_pipeline_submit")
        else:
            _check(load_library().zcg_pipeline_submit_wait(self.handle, a.ctypes.data, a.size,
                                                           int(timeout_ms), ctypes.byref(slot)),
                   "zcg_pipeline_submit_wait")
        return int(slot.value)

    def finish(self) -> None:
        _check(load_library().zcg_pipeline_finish(self.handle), "zcg_pipeline_finish")

    def next(self, timeout_ms: int = -1) -> Optional[int]:
        """Consumer: slot of the next submitted minibatch, None once the producer has finished
        and the ring is drained."""
        slot = ctypes.c_int(-1)
        rc = load_library().zcg_pipeline_next(self.handle, int(timeout_ms), ctypes.byref(slot))
        if rc == ECLOSED:
            return None
        _check(rc, "zcg_pipeline_next")
        return int(slot.value)

    def acquire(self, slot: int, consumer_stream=None):
        """Returns (buffer object given at creation, rows gathered into it)."""
        dev, n = ctypes.c_void_p(), ctypes.c_int64(0)
        _check(load_library().zcg_pipeline_acquire(self.handle, slot, _stream(consumer_stream),
                                                   ctypes.byref(dev), ctypes.byref(n)),
               "zcg_pipeline_acquire")
        return self._bufs[slot], int(n.value)

    def release(self, slot: int, consumer_stream=None) -> None:
        _check(load_library().zcg_pipeline_release(self.handle, slot, _stream(consumer_stream)),
               "zcg_pipeline_release")

    def close(self) -> None:
        if self.handle:
            h, self.handle = self.handle, 0
            _check(load_library().zcg_pipeline_destroy(h), "zcg_pipeline_destroy")


def pipeline_create(table: Table, max_rows: int, out_bufs, gather_stream=None) -> Pipeline:
    return Pipeline(table, max_rows, out_bufs, gather_stream)


def gather_ordered(table: Table, idx_dev, order_dev, out_dev, opts: Optional[LaunchOpts] = None,
                   n_idx: Optional[int] = None, stream=None) -> None:
    _check_idx_tensor(idx_dev)
    _check_idx_tensor(order_dev)
    rc = load_library().zcg_gather_ordered(table.handle, _ptr(idx_dev), _ptr(order_dev),
                                           _n_idx(idx_dev, n_idx), _ptr(out_dev), _stream(stream),
                                           ctypes.byref(opts) if opts is not None else None)
    _check(rc, "zcg_gather_ordered")


def order_workspace_bytes(n_idx: int) -> int:
    b = ctypes.c_int64(0)
    _check(load_library().zcg_order_workspace_bytes(n_idx, ctypes.byref(b)), "zcg_order_workspace_bytes")
    return int(b.value)


def gather_workspace_bytes(n_idx: int) -> int:
    b = ctypes.c_int64(0)
    _check(load_library().zcg_gather_workspace_bytes(n_idx, ctypes.byref(b)), "zcg_gather_workspace_bytes")
    return int(b.value)


def make_order(idx_dev, n_rows: int, order_dev, workspace_dev, workspace_bytes: int,
               n_idx: Optional[int] = None, stream=None) -> None:
    _check_idx_tensor(idx_dev)
    rc = load_library().zcg_make_order(_ptr(idx_dev), _n_idx(idx_dev, n_idx), n_rows, _ptr(order_dev),
                                       _ptr(workspace_dev), workspace_bytes, _stream(stream))
    _check(rc, "zcg_make_order")


STATIC_ORDER_MAX_IDX = 1 << 20


def make_order_static(idx_dev, n_rows: int, order_dev, n_idx: Optional[int] = None, stream=None) -> None:
    _check_idx_tensor(idx_dev)
    rc = load_library().zcg_make_order_static(_ptr(idx_dev), _n_idx(idx_dev, n_idx), n_rows,
                                              _ptr(order_dev), _stream(stream))
    _check(rc, "zcg_make_order_static")
