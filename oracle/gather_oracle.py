"""ctypes front end of ``gather_oracle.c`` (TEST INFRASTRUCTURE ONLY).

``gather(table, idx)`` returns ``out[i, :] = table[idx[i], :]`` (Section 3.2.1,
Listing 2 semantics) computed by the plain C loop, byte for byte.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gather_oracle.c")
_LIB_PATH = os.path.join(_HERE, "libgather_oracle.so")
_lib = None


class OracleRangeError(IndexError):
    """An index was outside [0, n_rows)."""


def build(verbose: bool = False) -> str:
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=gnu11", "-o", _LIB_PATH, _SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    global _lib
    _lib = None
    return _LIB_PATH


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.zcg_oracle_gather.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                          ctypes.c_int, ctypes.c_void_p]
        lib.zcg_oracle_gather.restype = ctypes.c_int
        _lib = lib
    return _lib


def gather_bytes(table_ptr: int, n_rows: int, row_bytes: int, idx: np.ndarray, out_ptr: int,
                 n_threads: int = 1) -> None:
    """Raw-pointer form: gathers into caller-owned memory at ``out_ptr``."""
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    bad = ctypes.c_int64(-1)
    rc = _load().zcg_oracle_gather(ctypes.c_void_p(table_ptr), n_rows, row_bytes,
                                   ctypes.c_void_p(idx.ctypes.data), idx.size,
                                   ctypes.c_void_p(out_ptr), n_threads, ctypes.byref(bad))
    if rc == -2:
        raise OracleRangeError(f"index at position {bad.value} is outside [0, {n_rows})")
    if rc != 0:
        raise ValueError("zcg_oracle_gather: bad arguments")


def gather(table: np.ndarray, idx: np.ndarray, n_threads: int = 1) -> np.ndarray:
    """``out[i, :] = table[idx[i], :]`` for a C-contiguous 2-D ``table``."""
    if table.ndim != 2 or not table.flags["C_CONTIGUOUS"]:
        raise ValueError("table must be a C-contiguous 2-D array")
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    if idx.ndim != 1:
        raise ValueError("idx must be 1-D")
    out = np.empty((idx.size, table.shape[1]), dtype=table.dtype)
    row_bytes = table.shape[1] * table.itemsize
    if row_bytes == 0:
        raise ValueError("rows must not be empty")
    gather_bytes(table.ctypes.data, table.shape[0], row_bytes, idx, out.ctypes.data, n_threads)
    return out
