"""Hand-written gfx950 code is not seen by the compiler's hazard recogniser.  On this chip a lane read
(v_readfirstlane / v_readlane) must not directly follow the VALU instruction that writes the register it
reads (one wait state); this test reads the inline assembly of the HIP sources and checks that rule."""
import os
import re

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2406_06237_amd", "csrc")


def _asm_instructions(text):
    """Instructions of all inline-assembly string literals, in source order: (line number, mnemonic, operands)."""
    out = []
    for no, line in enumerate(text.splitlines(), 1):
        for lit in re.findall(r'"((?:[^"\\]|\\.)*)"', line):
            for ins in lit.replace("\\t", " ").split("\\n"):
                ins = ins.strip()
                m = re.match(r"^([vs]_[a-z0-9_]+|ds_[a-z0-9_]+|global_[a-z0-9_]+)\s*(.*)$", ins)
                if m:
                    out.append((no, m.group(1), m.group(2)))
    return out


def _vgprs(operand):
    operand = operand.strip()
    m = re.match(r"^v\[(\d+):(\d+)\]$", operand)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"^v(\d+)$", operand)
    return {int(m.group(1))} if m else set()


def test_no_lane_read_directly_behind_the_write_of_its_register():
    checked = 0
    for name in sorted(os.listdir(CSRC)):
        if not name.endswith(".hip"):
            continue
        ins = _asm_instructions(open(os.path.join(CSRC, name)).read())
        for i, (no, op, args) in enumerate(ins):
            if not op.startswith(("v_readfirstlane", "v_readlane")):
                continue
            checked += 1
            read = _vgprs(args.split(",")[1]) if "," in args else set()
            if not read or i == 0:
                continue                      # an operand the compiler names: several instructions stand before it
            prev_no, prev_op, prev_args = ins[i - 1]
            if prev_op.startswith("v_"):
                written = _vgprs(prev_args.split(",")[0])
                assert not (written & read), f"{name}:{no}: {op} {args} directly behind {prev_op} {prev_args}"
    assert checked >= 4                       # the look-ahead kernel's block reads lanes in its loop and its wait
