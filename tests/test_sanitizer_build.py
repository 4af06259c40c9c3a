"""The host planner, the plan store, the host replay of the kernels' index arithmetic and the C oracle, built
with AddressSanitizer and UndefinedBehaviorSanitizer (g++/gcc, no HIP, no GPU) and run through
tests/sanitizer_driver.cpp: a planner that reads or writes out of bounds, overflows a signed integer or
shifts too far fails here instead of on the GPU."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1603_02297_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    oracle_o = str(tmp_path / "oracle.o")
    exe = str(tmp_path / "sanitizer_driver")
    subprocess.run(["gcc", "-std=c11", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra", *SAN,
                    "-c", os.path.join(ROOT, "oracle", "ttc_oracle.c"), "-o", oracle_o], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wno-unused-function", "-Wno-unknown-pragmas", *SAN,
                    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                    os.path.join(ROOT, "tests", "sanitizer_driver.cpp"),
                    os.path.join(CSRC, "ttc_plan.cpp"), os.path.join(CSRC, "ttc_cache.cpp"), oracle_o,
                    "-static-libasan", "-fopenmp", "-lm", "-o", exe], check=True)
    env = dict(os.environ, TMPDIR=str(tmp_path), ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0, res.stdout[-4000:] + res.stderr[-4000:]
    assert "sanitizer driver ok" in res.stdout
