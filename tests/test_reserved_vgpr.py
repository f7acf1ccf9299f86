"""The encode kernels keep one VGPR out of the compiler's hands for the ticket that is in flight
across iterations (see ticket_request in csrc/kernels.hip).  This compiles the kernels to assembly
and checks that nothing but the two hand-written instructions ever names that register, and that
the kernels neither spill nor exceed their register budget: a compiler that ignored the reservation
would corrupt tickets silently."""
import os
import re
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_06534_amd", "csrc")


def kernel_bodies(asm):
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


def test_reserved_register_is_only_named_by_the_ticket_routines():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as tmp:
        s_path = os.path.join(tmp, "kernels.s")
        subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                               "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"),
                               "-I", CSRC, "--cuda-device-only", "-S", os.path.join(CSRC, "kernels.hip"), "-o", s_path],
                              stderr=subprocess.DEVNULL)
        asm = open(s_path).read()
    bodies = kernel_bodies(asm)
    assert set(bodies) == {(f, r, a) for f in (0, 1) for r in (0, 1) for a in (0, 1)}
    for (f32, refresh, arith), body in bodies.items():
        reg = 255 if (f32 and refresh and arith) else 167 if (f32 or (refresh and arith)) else 127
        budget = reg + 1
        uses = 0
        for line in body:
            code = line.split(";")[0]
            if not code.strip() or code.strip().startswith("."):
                continue
            for m in re.finditer(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]", code):
                lo = int(m.group(1)) if m.group(1) else int(m.group(2))
                hi = int(m.group(1)) if m.group(1) else int(m.group(3))
                assert hi < budget, (f32, refresh, arith, code)
                if lo == hi == reg - 1 and re.match(r"\s*v_(writelane|readlane)_b32\b", code):
                    continue        # the register below it: the compiler may park scalar registers there
                if lo <= reg <= hi or lo <= reg - 1 <= hi:
                    # the reserved register (and the one below it otherwise) may only appear in the asm routines
                    assert re.search(r"global_atomic_add v%d, " % reg, code) or re.search(r"v_mov_b32 v\d+, v%d\s*$" % reg, code), \
                        (f32, refresh, arith, code)
                    uses += 1
            assert "scratch_" not in code, (f32, refresh, arith, code)
        assert uses >= 4, (f32, refresh, arith, uses)      # requests and takes are there
