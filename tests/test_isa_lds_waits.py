"""Static check of the assembly hipcc generates for this build's own kernels (CPU machine, no GPU).

The tile kernels read LDS from inline assembly (ds_read_b128 / ds_read_b64_tr_b16) and wait for the
data with hand-placed `s_waitcnt lgkmcnt(N)`: the compiler does not know that the destination
registers are invalid until that wait.  It is free to copy such a register, or to reuse it, between
the read and the wait -- it did once, in one of two instances of the same source, after a branch had
come to lie between them.  This test walks every kernel of the three sources in program order, keeps
the LDS/scalar-memory operations in flight as the counter sees them, and fails on any instruction
that touches the destination of an assembly read that no wait has covered yet."""
import re

import pytest

from paper_2508_15881_amd import build as b

SOURCES = ["decode_mfma.hip", "prefill_mfma.hip", "absorb_combine_mfma.hip"]
_REG = re.compile(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b")
_LGKM_OP = re.compile(r"^(ds_|s_load|s_buffer_load|s_memtime|s_memrealtime)")


def _vgprs(text):
    regs = set()
    for m in _REG.finditer(text):
        if m.group(3) is not None:
            regs.add(int(m.group(3)))
        else:
            regs.update(range(int(m.group(1)), int(m.group(2)) + 1))
    return regs


def _kernels(asm):
    """name -> list of (instruction text, inside inline assembly?) in program order."""
    out, cur, in_asm = {}, None, False
    for line in asm.splitlines():
        m = re.match(r"^(_ZN4tpla\w+):", line)
        if m:
            cur, in_asm = m.group(1), False
            out[cur] = []
            continue
        if cur is None:
            continue
        t = line.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        t = t.split(";")[0].strip()
        if not t or t.startswith(".") or t.endswith(":"):
            continue
        out[cur].append((t, in_asm))
        if t == "s_endpgm":
            cur = None
    return out


def check_kernel(insts):
    """Returns the violations of one kernel: (index, instruction, registers touched too early)."""
    in_flight = []          # operations the lgkm counter still counts, oldest first: set of unsafe destination registers
    bad = []
    for i, (t, in_asm) in enumerate(insts):
        mnem = t.split()[0]
        if mnem == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", t)
            if m:
                n = int(m.group(1))
                in_flight = in_flight[len(in_flight) - n:] if n else []
            elif "vmcnt" not in t and "expcnt" not in t:
                in_flight = []                       # a bare numeric s_waitcnt: treated as a full wait
            continue
        unsafe = set().union(*in_flight) if in_flight else set()
        operands = t[len(mnem):]
        touched = _vgprs(operands) & unsafe
        if touched:
            bad.append((i, t, sorted(touched)))
        if _LGKM_OP.match(mnem):
            dest = set()
            if in_asm and mnem.startswith("ds_read"):
                dest = _vgprs(operands.split(",")[0])       # the compiler has no wait of its own for these
            in_flight.append(dest)
    return bad


def test_the_checker_sees_a_copy_before_the_wait():
    """The failure this test exists for, as a four-line kernel: a copy of the read's destination ahead of
    the wait is reported, the same copy after the wait is not."""
    early = [("ds_read_b128 v[150:153], v142", True), ("v_mov_b64_e32 v[168:169], v[152:153]", False),
             ("s_waitcnt lgkmcnt(0)", True), ("v_add_f32_e32 v1, v150, v2", False)]
    late = [early[0], early[2], early[1], early[3]]
    assert [v[1] for v in check_kernel(early)] == ["v_mov_b64_e32 v[168:169], v[152:153]"]
    assert check_kernel(late) == []
    # a partial wait covers the oldest reads only
    ring = [("ds_read_b128 v[10:13], v1", True), ("ds_read_b128 v[14:17], v1 offset:128", True), ("s_waitcnt lgkmcnt(1)", True),
            ("v_mfma_f32_16x16x32_bf16 v[0:3], v[10:13], v[20:23], v[0:3]", False),
            ("v_mfma_f32_16x16x32_bf16 v[0:3], v[14:17], v[20:23], v[0:3]", False)]
    assert [v[0] for v in check_kernel(ring)] == [4]


# the third entry: the 32-heads-per-wave instances, which only exist in the measurement build
@pytest.mark.parametrize("source,flags", [(s, ()) for s in SOURCES] + [("decode_mfma.hip", ("-DTPLA_H32",))],
                         ids=SOURCES + ["decode_mfma.hip-H32"])
def test_no_instruction_touches_an_lds_read_before_its_wait(source, flags):
    kernels = _kernels(b.device_assembly(source, flags))
    assert kernels, source
    n_reads = 0
    for name, insts in kernels.items():
        n_reads += sum(1 for t, in_asm in insts if in_asm and t.startswith("ds_read"))
        bad = check_kernel(insts)
        assert not bad, "%s: %d instruction(s) use the destination of an LDS read before a wait covers it, first: %r" % (
            name, len(bad), bad[0])
    assert n_reads >= 16, "hardly any assembly LDS reads found in %s: has the listing format changed?" % source
