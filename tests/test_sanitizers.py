"""The CPU oracle and the library's host-side helpers under AddressSanitizer and
UndefinedBehaviorSanitizer (host code only; no GPU): tests/sanitize_driver.cpp is built together with
oracle/fspad_oracle.c and csrc/fspad_host.cpp and run on seeded small cases."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_and_host_helpers_are_clean_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
    oracle_obj = str(tmp_path / "oracle.o")
    exe = str(tmp_path / "sanitize_driver")
    subprocess.run(["gcc", "-std=c11", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra", "-c"] + san +
                   ["-o", oracle_obj, os.path.join(ROOT, "oracle", "fspad_oracle.c")], check=True)
    subprocess.run(["g++", "-std=c++17", "-fopenmp", "-static-libasan", "-Wall"] + san +
                   ["-I", os.path.join(ROOT, "include"), "-o", exe, os.path.join(ROOT, "tests", "sanitize_driver.cpp"),
                    os.path.join(ROOT, "paper_2408_15562_amd", "csrc", "fspad_host.cpp"), oracle_obj, "-lm"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="3")
    proc = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert proc.returncode == 0, proc.stdout + proc.stderr
    assert "runtime error" not in proc.stderr and "AddressSanitizer" not in proc.stderr, proc.stderr
    assert "sanitize_driver: clean" in proc.stdout
