"""Builds libzcgather.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libzcgather.so")
SOURCES = ["zcg_kernels.hip", "zcg_api.hip", "zcg_cpu_baseline.hip", "zcg_pipeline.hip"]


def hipcc_command() -> list:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return [
        hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-pthread",
        # keep the compiler from forming packed-fp32 instructions (none are wanted here;
        # this is byte movement, but the flag is the house rule for all device code)
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
        "-o", LIB_PATH,
    ] + [os.path.join(HERE, "csrc", s) for s in SOURCES]


def build(verbose: bool = False) -> str:
    cmd = hipcc_command()
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"
    out = "\n".join(l for l in proc.stdout.splitlines() if noise not in l and l.strip())
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    if verbose and out:
        print(out, flush=True)
    return LIB_PATH


if __name__ == "__main__":
    build(verbose=True)
