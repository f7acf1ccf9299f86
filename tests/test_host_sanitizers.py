"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the CPU oracle and the planner
are built with gcc / g++ and -fsanitize=address,undefined together with small drivers
(tests/sanitize/) and run as separate programs.  A report from either sanitizer ends the program
with a non-zero status."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"]


def run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)                      # the sanitizer runtime has to be the first one loaded
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout[-4000:]


def test_oracle_under_sanitizers():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "oracle_driver")
        subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra"] + SAN +
                              [os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
                               os.path.join(ROOT, "oracle", "rose_oracle.c"), "-lm", "-o", exe])
        run(exe)


def test_planner_under_sanitizers():
    csrc = os.path.join(ROOT, "paper_2605_06534_amd", "csrc")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "plan_driver")
        subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra", "-pthread"] + SAN +
                              ["-I", os.path.join(ROOT, "include"), "-I", csrc,
                               os.path.join(ROOT, "tests", "sanitize", "plan_driver.cpp"),
                               os.path.join(csrc, "plan.cpp"), "-o", exe])
        run(exe)
