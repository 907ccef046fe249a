"""A host-resident tensor that the GPU indexes directly (the paper's "unified tensor", Section 3.1,
Listing 1): ``u = to_unified(cpu_tensor); rows = u[idx_cuda]``.

Plumbing only: it owns a table handle, allocates the output with torch and calls the C ABI; the
gather itself runs in the library's kernels. Two ways to make the host memory GPU-visible:
``pin="copy"`` (default) allocates pinned mapped memory and copies the data in once at set-up;
``pin="register"`` pins the caller's own memory in place (no copy, the paper's route), where the
platform allows ``hipHostRegister``.
"""
from __future__ import annotations

import ctypes
from typing import Optional

import numpy as np

from . import binding as _b

_SIZE_TO_DTYPE = {1: _b.B8, 2: _b.F16, 4: _b.F32, 8: _b.B64}


class UnifiedTensor:
    def __init__(self, table: _b.Table, torch_dtype, shape, keepalive=None):
        self.table, self.dtype, self.shape = table, torch_dtype, tuple(shape)
        self._keepalive = keepalive  # the caller's array when it was pinned in place
        self._workspace = None       # device scratch lent to the gather (short-row tables only)

    def gather(self, idx, out=None, stream=None, ordered_by=None):
        """rows = self[idx]; ``idx`` is a 1-D int64 CUDA tensor, ``out`` an optional CUDA tensor."""
        import torch

        if idx.dim() != 1:
            raise ValueError("index list must be 1-D")
        if out is None:
            out = torch.empty((idx.numel(), self.shape[1]), dtype=self.dtype, device=idx.device)
        elif out.dtype != self.dtype or tuple(out.shape) != (idx.numel(), self.shape[1]) \
                or not out.is_contiguous():
            raise ValueError("out must be a contiguous [len(idx), dim] tensor of the table's dtype")
        stream = stream if stream is not None else torch.cuda.current_stream(idx.device)
        if ordered_by is not None:
            _b.gather_ordered(self.table, idx, ordered_by, out, stream=stream)
        elif self.table.row_bytes <= 128 and idx.numel() >= 32768:
            # rows of at most a line: lend the library scratch memory (torch's allocator, grown to
            # the longest list seen, reused from call to call) so that it can walk long dense
            # lists in ascending table order. One workspace per tensor: callers that gather from
            # one unified tensor on several streams at once pass their own ``out`` and order.
            need = _b.gather_workspace_bytes(idx.numel())
            if self._workspace is None or self._workspace.numel() < need:
                self._workspace = torch.empty(need, dtype=torch.uint8, device=idx.device)
            opts = _b.LaunchOpts(workspace_dev=self._workspace.data_ptr(), workspace_bytes=self._workspace.numel())
            _b.gather_ex(self.table, idx, out, opts, stream=stream)
        else:
            _b.gather(self.table, idx, out, stream=stream)
        return out

    def __getitem__(self, idx):
        return self.gather(idx)

    def host_view(self) -> np.ndarray:
        """numpy view of the host memory as raw elements of the table's element size."""
        return self.table.host_array()

    def close(self) -> None:
        self.table.close()
        self._keepalive = None
        self._workspace = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def to_unified(t, device: int = 0, pin: str = "copy", flags: int = _b.ALLOC_DEFAULT) -> UnifiedTensor:
    """Make a 2-D CPU torch tensor (or numpy array) indexable by the GPU without moving it to HBM."""
    import torch

    if isinstance(t, np.ndarray):
        t = torch.from_numpy(t)
    if t.device.type != "cpu" or t.dim() != 2 or not t.is_contiguous():
        raise ValueError("expected a contiguous 2-D CPU tensor")
    dt = _SIZE_TO_DTYPE.get(t.element_size())
    if dt is None:
        raise TypeError(f"unsupported element size {t.element_size()}")
    n_rows, dim = t.shape
    if pin == "register":
        table = _b.register_table(t.data_ptr(), n_rows, dim, dt, device)
        return UnifiedTensor(table, t.dtype, t.shape, keepalive=t)
    if pin != "copy":
        raise ValueError('pin must be "copy" or "register"')
    table = _b.alloc_table(n_rows, dim, dt, flags, device)
    ctypes.memmove(table.host_ptr, t.data_ptr(), n_rows * dim * t.element_size())
    return UnifiedTensor(table, t.dtype, t.shape)
