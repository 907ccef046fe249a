"""Host code under AddressSanitizer + UBSan: the C oracle and the input generators."""
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
