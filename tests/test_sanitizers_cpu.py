"""AddressSanitizer + UndefinedBehaviorSanitizer over the host-side C++ (the oracle and the worker
pool with the synthetic environment): both are built with -fsanitize=address,undefined into one
driver program (tests/sanitize/driver.cpp) that calls their entry points on small inputs, including
the supplied-ReLU-decision mode, both storage modes, the value-based variant, and out-of-range
actions for the environment.  CPU only; no GPU code is involved."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_and_worker_pool_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_driver")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-fopenmp", "-pthread", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           os.path.join(ROOT, "tests", "sanitize", "driver.cpp"), os.path.join(ROOT, "oracle", "paac_oracle.cpp"),
           os.path.join(ROOT, "paper_1705_04862_amd", "csrc", "actors.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitizer driver ok" in r.stdout
