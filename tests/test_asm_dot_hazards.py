"""Host-side check of the kernels' machine code: dot products written as assembly statements.

On gfx950 an instruction of another kind that reads the result of a dot product needs three wait
states after it; a dot product that takes the result as its addend may follow at once.  The
compiler keeps that distance for the dot products it emits itself but cannot see inside an assembly
statement, so the sources promise it by construction (the result feeds only another dot product's
addend, or the statement ends with s_nop 2).  This test compiles the kernels to assembly and checks
the promise on every such instruction of every instantiation.  No GPU needed."""
import os
import re
import subprocess

from paper_2407_00088_amd import build as B

FILES = ["tmac_perm.hip", "tmac_kernels.hip", "tmac_rows.hip"]
DOT = re.compile(r"(v_dot2_f32_f16|v_dot4_i32_i8) (v\d+),")


def instructions(path):
    """(text, written inside an assembly statement) per instruction; labels as ('LABEL', False)."""
    out, in_asm = [], False
    for line in open(path):
        t = line.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
        elif t.startswith(";;#ASMEND"):
            in_asm = False
        elif t.endswith(":") and not t.startswith(";"):
            out.append(("LABEL", False))
        elif re.match(r"^(v_|s_|ds_|global_|buffer_|flat_|scratch_)", t):
            out.append((t.split(";")[0].strip(), in_asm))
    return out


def first_reader(ins, i, reg):
    """('addend' | 'other' | None, wait states before it) for the first instruction after ins[i] that reads reg."""
    ws = 0
    for text, _ in ins[i + 1:i + 80]:
        if text == "LABEL":
            return None, ws
        op, _, rest = text.partition(" ")
        ops = [x.strip() for x in rest.split(",")]
        if op == "s_nop":
            ws += int(ops[0]) + 1
            continue
        in_place = op in ("v_dot2c_f32_f16_e32", "v_dot4c_i32_i8_e32") and ops[0] == reg  # dst is the addend
        if reg in ops[1:] or in_place:
            as_addend = op.startswith("v_dot") and (in_place and reg not in ops[1:] or not in_place and ops[-1] == reg
                                                    and reg not in ops[1:-1])
            return ("addend" if as_addend else "other"), ws
        if ops and ops[0] == reg:
            return None, ws  # overwritten unread
        ws += 1
    return None, ws


def test_assembly_dot_products_keep_their_distance(tmp_path):
    flags = [f for f in B.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    procs = []
    for f in FILES:
        out = tmp_path / (f + ".s")
        procs.append((out, subprocess.Popen([hipcc, *flags, "--offload-device-only", "-S", "-o", str(out),
                                             os.path.join(B.CSRC, f)], stderr=subprocess.DEVNULL)))
    seen = 0
    for out, pr in procs:
        assert pr.wait() == 0, out
        ins = instructions(out)
        for i, (text, in_asm) in enumerate(ins):
            m = DOT.match(text) if in_asm else None
            if not m:
                continue
            kind, ws = first_reader(ins, i, m.group(2))
            seen += 1
            assert kind in (None, "addend") or ws >= 3, (out.name, text, kind, ws)
    assert seen > 500   # the statements are there (the decode kernels alone hold over a thousand)


def test_the_checker_tells_an_addend_from_another_reader(tmp_path):
    """Planted cases: the result read at once by a dot product as its addend (fine), by another kind
    of instruction one wait state later (flagged), and by that instruction after s_nop 2 (fine)."""
    src = """
	;;#ASMSTART
	v_dot2_f32_f16 v39, v39, s46, 0
	;;#ASMEND
	v_dot2c_f32_f16_e32 v39, 0x3c003c00, v19
	;;#ASMSTART
	v_dot2_f32_f16 v38, v38, s46, v39
	;;#ASMEND
	v_and_b32_e32 v40, 0x7fff7fff, v21
	v_max3_f32 v38, v38, 0, v39
	;;#ASMSTART
	v_dot2_f32_f16 v1, v2, s46, 0
	s_nop 2
	;;#ASMEND
	v_add_f32_e32 v3, v1, v1
	;;#ASMSTART
	v_dot4_i32_i8 v5, v6, v7, 0
	;;#ASMEND
	v_dot4c_i32_i8_e32 v5, v8, v9
"""
    f = tmp_path / "planted.s"
    f.write_text(src)
    ins = instructions(f)
    got = [first_reader(ins, i, DOT.match(t).group(2)) for i, (t, a) in enumerate(ins) if a and DOT.match(t)]
    assert got == [("addend", 0), ("other", 1), ("other", 3), ("addend", 0)]
