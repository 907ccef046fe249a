"""Host code under AddressSanitizer + UBSan: the C oracle, the input generators, and the gather
library's launch planning (pure host arithmetic that decides what the kernels are launched with)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_and_generators_are_clean_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_driver")
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-std=gnu11", "-o", exe, os.path.join(ROOT, "tests", "sanitize_driver.c"),
           os.path.join(ROOT, "oracle", "gather_oracle.c"),
           os.path.join(ROOT, "zcg_workload", "csrc", "workload.c"), "-lm"]
    subprocess.run(cmd, check=True)
    # other preloaded libraries may sit before the sanitizer runtime: do not insist on the order
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               OMP_NUM_THREADS="4")
    proc = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env,
                          timeout=120)
    assert proc.returncode == 0 and "sanitize driver ok" in proc.stdout, proc.stdout[-3000:]


def test_launch_planning_is_clean_under_asan_ubsan(tmp_path):
    """zcg_plan.hip holds no device code: built as plain C++ with g++ and driven over 200,000 seeded
    combinations of shapes, addresses, list lengths and options, extreme values included."""
    exe = str(tmp_path / "sanitize_plan_driver")
    csrc = os.path.join(ROOT, "paper_2103_03330_amd", "csrc")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include", "-I", os.path.join(ROOT, "include"), "-I", csrc,
           "-o", exe, os.path.join(ROOT, "tests", "sanitize_plan_driver.cpp"), "-x", "c++",
           os.path.join(csrc, "zcg_plan.hip")]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    proc = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert proc.returncode == 0 and "plan driver ok" in proc.stdout, proc.stdout[-3000:]
