"""Builds libzcgather.so (HIP kernels + C ABI) and libzcgprobe.so (measurement probes for the
benchmark and the tests) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libzcgather.so")
PROBE_LIB_PATH = os.path.join(HERE, "libzcgprobe.so")
SOURCES = ["zcg_kernels.hip", "zcg_plan.hip", "zcg_api.hip", "zcg_cpu_baseline.hip", "zcg_pipeline.hip",
           "zcg_order.hip"]
PROBE_SOURCES = ["zcg_probe.hip"]


BUILD_DIR = os.path.join(HERE, "_build")
NOISE = "is not a recognized feature for this target"


def hipcc_flags() -> list:
    return [
        "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-pthread",
        # keep the compiler from forming packed-fp32 instructions (none are wanted here;
        # this is byte movement, but the flag is the house rule for all device code)
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
    ]


def build(verbose: bool = False) -> str:
    """Compile every translation unit (in parallel) and link the two shared objects."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(BUILD_DIR, exist_ok=True)
    procs = []
    for src in SOURCES + PROBE_SOURCES:
        obj = os.path.join(BUILD_DIR, src + ".o")
        cmd = [hipcc] + hipcc_flags() + ["-c", "-o", obj, os.path.join(HERE, "csrc", src)]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE,
                                                 stderr=subprocess.STDOUT, text=True)))
    objs = {}
    for src, obj, proc in procs:
        out, _ = proc.communicate()
        if proc.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n" + out)
        out = "\n".join(l for l in out.splitlines() if NOISE not in l and l.strip())
        if verbose and out:
            print(out, flush=True)
        objs[src] = obj
    for path, srcs in ((LIB_PATH, SOURCES), (PROBE_LIB_PATH, PROBE_SOURCES)):
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", "-o", path] + \
            [objs[s] for s in srcs]
        if verbose:
            print(" ".join(link), flush=True)
        proc = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if proc.returncode != 0:
            raise RuntimeError("link failed:\n" + proc.stdout)
    return LIB_PATH


if __name__ == "__main__":
    build(verbose=True)
