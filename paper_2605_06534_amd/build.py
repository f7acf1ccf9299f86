"""Build librose_delta.so for gfx950 with hipcc (in-tree, next to this file)."""
import os
import re
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librose_delta.so")
SOURCES = ["plan.cpp", "api.cpp", "kernels.hip"]


DEVICE_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _encode_kernel_bodies(asm):
    out, name, body = {}, None, []
    for line in asm.splitlines():
        m = re.match(r"^(_ZN4rose13encode_kernelILi(\d)ELi(\d)ELi(\d)EEEvNS_10EncodeArgsE):", line)
        if m:
            name, body = (int(m.group(2)), int(m.group(3)), int(m.group(4))), []
            continue
        if name is not None:
            if line.startswith(".Lfunc_end"):
                out[name] = body
                name = None
            else:
                body.append(line)
    return out


def check_reserved_vgpr(extra=()):
    """The encode kernels keep one VGPR out of the compiler's hands for the ticket that is in flight
    across iterations (see ticket_request in csrc/kernels.hip); the compiler is only ASKED to stay below
    it.  Compile the kernels to assembly and make sure that nothing but the two hand-written
    instructions ever names that register, that no kernel exceeds its register budget and that none
    spills: a toolchain or flag change that broke the reservation would hand out corrupt tickets.
    Raises RuntimeError on a violation."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as tmp:
        s_path = os.path.join(tmp, "kernels.s")
        subprocess.check_call([hipcc] + DEVICE_FLAGS + list(extra) +
                              ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "--cuda-device-only", "-S",
                               os.path.join(CSRC, "kernels.hip"), "-o", s_path], stderr=subprocess.DEVNULL)
        with open(s_path) as f:
            asm = f.read()
    bodies = _encode_kernel_bodies(asm)
    if set(bodies) != {(f, r, a) for f in (0, 1) for r in (0, 1) for a in (0, 1)}:
        raise RuntimeError("not all eight encode kernels were found in the assembly: %s" % sorted(bodies))
    for (f32, refresh, arith), body in sorted(bodies.items()):
        reg = 255 if (f32 and refresh and arith) else 167 if (f32 or (refresh and arith)) else 127
        budget, uses, what = reg + 1, 0, "encode_kernel<%d, %d, %d>" % (f32, refresh, arith)
        for line in body:
            code = line.split(";")[0]
            if not code.strip() or code.strip().startswith("."):
                continue
            for m in re.finditer(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]", code):
                lo = int(m.group(1)) if m.group(1) else int(m.group(2))
                hi = int(m.group(1)) if m.group(1) else int(m.group(3))
                if hi >= budget:
                    raise RuntimeError("%s goes past its register budget: %s" % (what, code.strip()))
                if lo == hi == reg - 1 and re.match(r"\s*v_(writelane|readlane)_b32\b", code):
                    continue        # the register below it: the compiler may park scalar registers there
                if lo <= reg <= hi or lo <= reg - 1 <= hi:
                    # the reserved register (and otherwise the one below it) may only appear in the asm routines
                    if not (re.search(r"global_atomic_add v%d, " % reg, code) or
                            re.search(r"v_mov_b32 v\d+, v%d\s*$" % reg, code)):
                        raise RuntimeError("%s: the compiler uses the reserved register: %s" % (what, code.strip()))
                    uses += 1
            if "scratch_" in code:
                raise RuntimeError("%s spills: %s" % (what, code.strip()))
        if uses < 4:
            raise RuntimeError("%s: the ticket routines are missing (%d uses of v%d)" % (what, uses, reg))


def build(verbose=False, extra=(), out=None, check=True):
    """Compile the library; with check (the default) also verify the reserved-register assumption of
    the encode kernels and refuse to leave a library behind that breaks it."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if check:
        check_reserved_vgpr(extra)
    cmd = [hipcc] + DEVICE_FLAGS + ["-fPIC", "-shared", "-Wall", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd += list(extra)
    for s in SOURCES:
        if s.endswith(".cpp"):
            cmd += ["-x", "hip", os.path.join(CSRC, s)]
        else:
            cmd += [os.path.join(CSRC, s)]
    cmd += ["-o", out or LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return out or LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
