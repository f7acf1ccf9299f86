"""The boundary from plain C: include/rose_delta.h compiles as C99 and as C++11 with -pedantic, and
a C program linked against the built library plans a small parameter set and checks the host-side
queries (no GPU is touched)."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INC = os.path.join(ROOT, "include")
LIBDIR = os.path.join(ROOT, "paper_2605_06534_amd")


def test_header_is_plain_c_and_cxx():
    with tempfile.TemporaryDirectory() as tmp:
        src = os.path.join(tmp, "hdr.c")
        with open(src, "w") as f:
            f.write('#include "rose_delta.h"\nint main(void) { rose_tensor_desc t; (void)t; return (int)ROSE_OK; }\n')
        subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", INC, "-fsyntax-only", src])
        subprocess.check_call(["g++", "-std=c++11", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", INC, "-fsyntax-only",
                               "-x", "c++", src])


def test_plan_queries_from_a_c_program():
    assert os.path.exists(os.path.join(LIBDIR, "librose_delta.so")), "build the library first"
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "plan_from_c")
        subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-I", INC,
                               os.path.join(ROOT, "tests", "c_abi", "plan_from_c.c"),
                               "-L", LIBDIR, "-lrose_delta", "-Wl,-rpath," + LIBDIR, "-o", exe])
        r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
        assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout
