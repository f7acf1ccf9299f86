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


def test_binding_constants_are_the_headers():
    """The Python binding restates the header's numbers; a C program prints the header's, and the two
    must agree (a constant changed on one side only would otherwise pass silently)."""
    from paper_2605_06534_amd import binding
    from workloads import models
    names = {"ROSE_MAX_TP": binding.ROSE_MAX_TP, "ROSE_MAX_SECTIONS": binding.ROSE_MAX_SECTIONS,
             "ROSE_OK": binding.OK, "ROSE_ERR_ARG": binding.ERR_ARG, "ROSE_ERR_SHAPE": binding.ERR_SHAPE,
             "ROSE_ERR_CAPACITY": binding.ERR_CAPACITY, "ROSE_ERR_ALIGN": binding.ERR_ALIGN, "ROSE_ERR_HIP": binding.ERR_HIP,
             "ROSE_ERR_UNSUPPORTED": binding.ERR_UNSUPPORTED, "ROSE_ERR_SCRATCH": binding.ERR_SCRATCH,
             "ROSE_REPLICATED": binding.REPLICATED, "ROSE_SPLIT_ROWS": binding.SPLIT_ROWS, "ROSE_SPLIT_COLS": binding.SPLIT_COLS,
             "ROSE_FUSED_ROWS": binding.FUSED_ROWS, "ROSE_BF16": binding.BF16, "ROSE_FP32_RNE": binding.FP32_RNE,
             "ROSE_TILE_ORDER_AUTO_PICK": binding.TILE_ORDER_AUTO, "ROSE_TILE_ORDER_SPREAD": binding.TILE_ORDER_SPREAD,
             "ROSE_TILE_ORDER_NEIGHBOURS": binding.TILE_ORDER_NEIGHBOURS, "ROSE_TILE_ORDER_TIMED": binding.TILE_ORDER_TIMED,
             "ROSE_ENCODE_REFRESH": binding.ENCODE_REFRESH, "ROSE_ENCODE_ARITH": binding.ENCODE_ARITH,
             "ROSE_PAYLOAD_NEW": binding.PAYLOAD_NEW, "ROSE_PAYLOAD_ARITH": binding.PAYLOAD_ARITH,
             "ROSE_STATIC_SCRATCH_BYTES": binding.STATIC_SCRATCH_BYTES,
             "ROSE_LAYER_FIRST": models.LAYER_FIRST, "ROSE_LAYER_LAST": models.LAYER_LAST}
    with tempfile.TemporaryDirectory() as tmp:
        src, exe = os.path.join(tmp, "consts.c"), os.path.join(tmp, "consts")
        with open(src, "w") as f:
            f.write('#include <stdio.h>\n#include "rose_delta.h"\nint main(void) {\n')
            for n in names:
                f.write('    printf("%s %%lld\\n", (long long)(%s));\n' % (n, n))
            f.write("    return 0;\n}\n")
        subprocess.check_call(["gcc", "-std=c99", "-I", INC, src, "-o", exe])
        out = subprocess.run([exe], stdout=subprocess.PIPE, text=True, timeout=60).stdout
    got = dict((l.split()[0], int(l.split()[1])) for l in out.strip().splitlines())
    assert got == {k: int(v) for k, v in names.items()}
