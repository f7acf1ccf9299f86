"""The encode kernels keep one VGPR out of the compiler's hands for the ticket that is in flight
across iterations (see ticket_request in csrc/kernels.hip).  The build step compiles the kernels to
assembly and checks that nothing but the two hand-written instructions ever names that register,
and that the kernels neither spill nor exceed their register budget (a compiler that ignored the
reservation would corrupt tickets silently); this runs that check, and shows that it does notice a
kernel body that breaks the rules."""
import pytest

from paper_2605_06534_amd import build


def test_reserved_register_is_only_named_by_the_ticket_routines():
    build.check_reserved_vgpr()


def test_the_check_notices_violations(monkeypatch):
    good = ["\tglobal_atomic_add v127, v1, v2, s[0:1] sc0", "\tv_mov_b32 v5, v127"] * 2
    names = ["_ZN4rose13encode_kernelILi%dELi%dELi%dEEEvNS_10EncodeArgsE" % (f, r, a) for f in (0, 1) for r in (0, 1) for a in (0, 1)]

    def asm_with(first_body):
        out = []
        for i, n in enumerate(names):
            reg = 255 if n.count("Li1E") == 3 else 167 if ("ILi1E" in n or n.endswith("Li1ELi1EEEvNS_10EncodeArgsE")) else 127
            body = first_body if i == 0 else [l.replace("v127", "v%d" % reg) for l in good]
            out += [n + ":"] + body + [".Lfunc_end%d:" % i]
        return "\n".join(out)

    for bad_line, what in [("\tv_add_u32 v127, v1, v2", "reserved register"), ("\tv_add_u32 v200, v1, v2", "budget"),
                           ("\tscratch_store_dword off, v1, s0", "spills")]:
        bodies = build._encode_kernel_bodies(asm_with(good + [bad_line]))
        assert len(bodies) == 8
        monkeypatch.setattr(build.subprocess, "check_call", lambda *a, **k: 0)
        monkeypatch.setattr(build, "open", lambda *a, **k: __import__("io").StringIO(asm_with(good + [bad_line])), raising=False)
        with pytest.raises(RuntimeError) as e:
            build.check_reserved_vgpr()
        assert what in str(e.value), (what, str(e.value))
