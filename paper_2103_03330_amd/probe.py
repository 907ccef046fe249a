"""ctypes binding of libzcgprobe (``include/zcg_probe.h``): measurement probes for the benchmark
and the tests -- link peak, shader-issued read rate and latency of mapped host memory, a
known-size copy kernel, a stand-in compute kernel. Argument marshalling only; not part of the
gather."""
from __future__ import annotations

import ctypes
import os

from . import build as _build
from .binding import _ptr, _stream

EXPORTS = ["zcgp_last_hip_error", "zcgp_measure_h2d", "zcgp_measure_host_read_latency",
           "zcgp_measure_host_stream_read", "zcgp_device_copy", "zcgp_synthetic_compute"]

_lib = None


class ProbeError(RuntimeError):
    def __init__(self, status: int, what: str, hip_error: int = 0):
        self.status, self.hip_error = status, hip_error
        super().__init__(f"{what}: status {status}" + (f", hipError_t={hip_error}" if status == -4 else ""))


def load_library() -> ctypes.CDLL:
    """Load the built probe library; build first only if nothing is built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.PROBE_LIB_PATH):
        _build.build()
    lib = ctypes.CDLL(_build.PROBE_LIB_PATH)
    vp, i64, i32, pd = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.POINTER(ctypes.c_double)
    sigs = {
        "zcgp_last_hip_error": (i32, []),
        "zcgp_measure_h2d": (i32, [i64, i32, i32, pd]),
        "zcgp_measure_host_read_latency": (i32, [i32, i64, pd]),
        "zcgp_measure_host_stream_read": (i32, [i32, i64, i32, pd]),
        "zcgp_device_copy": (i32, [vp, vp, i64, vp]),
        "zcgp_synthetic_compute": (i32, [vp, i32, i64, vp]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _check(status: int, what: str) -> None:
    if status != 0:
        raise ProbeError(status, what, int(load_library().zcgp_last_hip_error()) if status == -4 else 0)


def measure_h2d(n_bytes: int, reps: int = 10, device: int = 0) -> float:
    """Median pinned host-to-device copy bandwidth in GB/s (1e9 bytes)."""
    g = ctypes.c_double(0.0)
    _check(load_library().zcgp_measure_h2d(n_bytes, reps, device, ctypes.byref(g)), "zcgp_measure_h2d")
    return float(g.value)


def measure_host_read_latency(hops: int = 20000, device: int = 0) -> float:
    """Round-trip time in microseconds of one dependent read of mapped host memory."""
    us = ctypes.c_double(0.0)
    _check(load_library().zcgp_measure_host_read_latency(device, hops, ctypes.byref(us)),
           "zcgp_measure_host_read_latency")
    return float(us.value)


def measure_host_stream_read(n_bytes: int = 256 << 20, reps: int = 10, device: int = 0) -> float:
    """GB/s at which GPU lanes stream consecutive bytes of mapped host memory into HBM."""
    g = ctypes.c_double(0.0)
    _check(load_library().zcgp_measure_host_stream_read(device, n_bytes, reps, ctypes.byref(g)),
           "zcgp_measure_host_stream_read")
    return float(g.value)


def device_copy(dst_dev, src_dev, n_bytes: int, stream=None) -> None:
    _check(load_library().zcgp_device_copy(_ptr(dst_dev), _ptr(src_dev), n_bytes, _stream(stream)),
           "zcgp_device_copy")


def synthetic_compute(stream, blocks: int, iters: int, sink_dev) -> None:
    _check(load_library().zcgp_synthetic_compute(_stream(stream), blocks, iters, _ptr(sink_dev)),
           "zcgp_synthetic_compute")
