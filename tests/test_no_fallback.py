"""The product path has no CPU fallback and never touches the oracle; the oracle never touches
the product. Checked statically on the sources and by taking the library away."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _sources(*dirs, exts=(".py", ".hip", ".h", ".c")):
    for d in dirs:
        for base, _, files in os.walk(os.path.join(ROOT, d)):
            if "_build" in base or "__pycache__" in base:
                continue
            for f in files:
                if f.endswith(exts):
                    yield os.path.join(base, f)


def test_product_and_oracle_do_not_know_each_other():
    uses_oracle = re.compile(r"^\s*(from|import)\s+oracle\b|gather_oracle|libgather_oracle", re.M)
    for path in _sources("paper_2103_03330_amd", "include", "zcg_workload"):
        assert not uses_oracle.search(open(path).read()), f"{path} refers to the oracle"
    uses_product = re.compile(r"paper_2103_03330_amd|zcgather|zcg_gather|hip/hip_runtime", re.M)
    for path in _sources("oracle"):
        assert not uses_product.search(open(path).read()), f"{path} refers to the HIP library"
    # the input generators hold none of the method: they name neither side
    for path in _sources("zcg_workload"):
        text = open(path).read()
        assert "paper_2103_03330_amd" not in text and "zcg_gather" not in text, path


def test_missing_library_raises_instead_of_falling_back():
    code = r"""
import numpy as np
import paper_2103_03330_amd as z
from paper_2103_03330_amd import binding, build
build.LIB_PATH = "/nonexistent/libzcgather.so"
def no_compiler(*a, **k):
    raise RuntimeError("no compiler here")
build.build = no_compiler
binding._lib = None
for call in (lambda: z.alloc_table(4, 4, "f32"),
             lambda: z.gather(z.Table(1, 4, 4, z.F32), np.zeros(1, np.int64), 0, n_idx=1),
             lambda: z.version()):
    try:
        call()
    except (RuntimeError, OSError) as exc:
        print("raised:", type(exc).__name__)
    else:
        raise SystemExit("a call succeeded without the library")
"""
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.count("raised:") == 3
