"""CPU oracle for the sparse feature gather -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline
leg may import this package. It shares no code with the GPU library and never
imports it.
"""
from .gather_oracle import build, gather, gather_bytes, OracleRangeError  # noqa: F401
