"""The rocprofv3 summaries under profiles/ must describe the kernels as they are now: the kernel
signature printed in the statistics matches the source, the counter summary carries the
fingerprint of the current kernel sources, and bench.py withholds traffic figures otherwise."""
import importlib.util
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# how the profiler prints the parameter types used in csrc/zcg_kernels.hip
PRINTED = {"const uint8_t*": "unsigned char const*", "const int64_t*": "long const*", "int64_t": "long",
           "uint8_t*": "unsigned char*", "int": "int", "unsigned": "unsigned int"}


def _bench():
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _source_signature(kernel):
    src = open(os.path.join(ROOT, "paper_2103_03330_amd", "csrc", "zcg_kernels.hip")).read()
    m = re.search(r"\b" + kernel + r"\(([^)]*)\)\s*\{", src)
    assert m, f"{kernel} not found in zcg_kernels.hip"
    types = []
    for param in m.group(1).split(","):
        param = param.replace("__restrict__", " ").strip()
        types.append(PRINTED[" ".join(param.split()[:-1])])
    return types


def test_kernel_statistics_name_the_kernels_of_the_source():
    text = open(os.path.join(ROOT, "profiles", "gather_cfg2_kernel_stats.txt")).read()
    seen = re.findall(r"(zcg_k_rows_\w+)<[^>]*>\(([^)]*)\)", text)
    assert any(name == "zcg_k_rows_wide_half" for name, _ in seen)  # config 2's default kernel
    for name, params in seen:
        assert [p.strip() for p in params.split(",")] == _source_signature(name), name


def test_counter_summary_carries_the_current_fingerprint_and_plan():
    bench = _bench()
    text = open(os.path.join(ROOT, "profiles", "gather_cfg2_counters.txt")).read()
    assert f"kernel_source_sha = {bench.kernel_source_sha()}" in text, \
        "the gather kernels changed after profiles/gather_cfg2_counters.txt was collected: collect it again"
    plan = {k: int(re.search(rf"^plan_{k} = (\d+)$", text, re.M).group(1)) for k in bench.PLAN_KEYS}
    got, note = bench.read_profile_traffic("gather_cfg2_counters.txt", plan)
    assert note is None and 400 < got["link_read_bytes_per_row"] < 520 and got["hbm_write_bytes_per_row"] >= 400
    # another launch plan, or a missing summary: no figures, and a reason
    other = dict(plan, blocks=plan["blocks"] // 2)
    got, note = bench.read_profile_traffic("gather_cfg2_counters.txt", other)
    assert got is None and "stale" in note and "plan_blocks" in note
    got, note = bench.read_profile_traffic("gather_cfg9_counters.txt", plan)
    assert got is None and note


def test_stale_fingerprint_is_refused(monkeypatch):
    bench = _bench()
    monkeypatch.setattr(bench, "kernel_source_sha", lambda: "0" * 16)
    got, note = bench.read_profile_traffic("gather_cfg2_counters.txt", {k: 0 for k in bench.PLAN_KEYS})
    assert got is None and "other kernel sources" in note
