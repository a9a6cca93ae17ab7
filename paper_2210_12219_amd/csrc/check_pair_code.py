#!/usr/bin/env python3
"""Build-time checks of the paired enumeration kernel's compiled code (run by build.py; fails the build loudly).

The kernel keeps the DP row in fixed registers across several inline-assembly blocks and jumps into generated code
at offsets computed from instruction sizes.  Both rest on what the toolchain emits, so both are verified on the
code it did emit:
  1. in the compiler's assembly of the kernel, no instruction outside the blocks touches a reserved register;
  2. in the disassembly of the assembled object, the instruction at every entry offset of ppo_pair_layout.json is
     the chain step or run step the table means (right chain, right depth, right registers), every header
     reads the table entry of the position below the code it follows, and the block ends where the table says.
"""
import json
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
KERNEL = "enumerate_paired_kernel"


def check_reserved_registers(asm_text, lay):
    lo, hi = lay["rb"], lay["vtop"]   # entry 0 has a (dummy) register too
    inside_kernel = in_asm = False
    seen_blocks = 0
    for n, line in enumerate(asm_text.splitlines(), 1):
        if re.match(rf"^_ZN3ppo\d+{KERNEL}\w*:", line):
            inside_kernel = True
            continue
        if not inside_kernel:
            continue
        if line.startswith(".Lfunc_end"):
            break
        if ";;#ASMSTART" in line:
            in_asm = True
            seen_blocks += 1
            continue
        if ";;#ASMEND" in line:
            in_asm = False
            continue
        if in_asm:
            continue
        code = line.split(";")[0]
        for m in re.finditer(r"\bv(\d+)\b", code):
            assert not lo <= int(m.group(1)) <= hi, f"line {n}: reserved register outside the blocks: {line.strip()}"
        for m in re.finditer(r"\bv\[(\d+):(\d+)\]", code):
            assert int(m.group(2)) < lo or int(m.group(1)) > hi, f"line {n}: reserved registers outside the blocks: {line.strip()}"
    assert inside_kernel and seen_blocks >= 6, "kernel or its blocks not found in the assembly"


def check_entry_offsets(disasm_text, lay):
    # instructions of the kernel by address
    instr, inside = {}, False
    for line in disasm_text.splitlines():
        if re.match(rf"^[0-9a-f]+ <_ZN3ppo\d+{KERNEL}\w*>:", line):
            inside = True
            continue
        if inside and re.match(r"^[0-9a-f]+ <", line):
            if re.match(r"^[0-9a-f]+ <ppo_pair_\w+>:", line):
                continue          # the blocks' own labels
            break
        if inside:
            m = re.match(r"^\s*(\S.*?)\s*//\s*([0-9A-Fa-f]+):", line)
            if m:
                instr[int(m.group(2), 16)] = re.sub(r"\s+", " ", m.group(1).strip())
    sb = lay["sbase"]
    bases = [a for a, t in instr.items() if t == f"s_getpc_b64 s[{sb}:{sb + 1}]"]
    assert len(bases) == 1, f"expected one base instruction, found {len(bases)}"
    base = bases[0] + 4
    rb, vacc, vinf = lay["rb"], lay["vacc"], lay["vinf"]
    R = lambda u: f"v{rb + u}"
    checked = 0
    for us, by_w in lay["entries"].items():
        u = int(us)
        for ws, off in by_w.items():
            w = int(ws)
            got = instr.get(base + off)
            if w == 0:
                want = f"v_mov_b32_e32 {R(u)}, v{vinf}"
            elif w & 1:
                J = (w - 1) // 2
                want = (f"v_pk_minimum3_f16 v{vacc}, v{vacc}, {R(u - 2 * J + 1)}, {R(u - 2 * J)}" if J
                        else f"v_pk_min_u16 {R(u)}, v{vacc}, {R(u)}")
            else:
                J = w // 2 - 1
                want = (f"v_pk_minimum3_f16 v{vacc}, v{vacc}, {R(u - 2 * J)}, {R(u - 2 * J - 1)}" if J
                        else f"v_pk_minimum3_f16 {R(u)}, v{vacc}, {R(u)}, {R(u - 1)}")
            assert got == want, f"entry u={u} w={w} at +{off}: found `{got}`, expected `{want}`"
            checked += 1
    # the run code: entered at position a of the piece ending at p, the first instruction folds entry a into the
    # output below it; the piece's header follows its last instruction
    for ps, by_a in lay["runs"].items():
        for as_, off in by_a.items():
            a = int(as_)
            got = instr.get(base + off)
            want = f"v_pk_min_u16 {R(a)}, {R(a - 1)}, {R(a)}"
            assert got == want, f"run code p={ps} a={a} at +{off}: found `{got}`, expected `{want}`"
            checked += 1
        p = int(ps)
        got = instr.get(base + by_a[ps] + 8)
        assert got == f"v_mov_b32_e32 v{vacc}, v{vinf}", f"no header after the run code ending at {p}: `{got}`"
    # every header reads the table entry of the position below the code it follows: the instruction after the
    # last one of a chain (8 bytes on) starts a header whose second instruction names that entry's register
    st0, nslot = lay["st0"], lay["nslot"]

    def header_reads(addr, position):
        slot = (position - 1) % nslot
        x, hi = slot // 2, slot & 1
        want = (f"s_lshr_b32 s{lay['stmp']}, s{st0 + x}, 16" if hi
                else f"s_and_b32 s{lay['stmp']}, s{st0 + x}, s{lay['smask']}")
        assert instr.get(addr) == f"v_mov_b32_e32 v{vacc}, v{vinf}" and instr.get(addr + 4) == want, \
            f"header for position {position} at +{addr - base}: `{instr.get(addr)}` / `{instr.get(addr + 4)}`, expected `{want}`"

    for us, by_w in lay["entries"].items():
        u = int(us)
        header_reads(base + by_w["1"] + 8, u - 1)    # after the odd chain's last instruction
        header_reads(base + by_w["0"] + 4, u - 1)    # after the +inf
        if "2" in by_w:
            header_reads(base + by_w["2"] + 8, u - 1)
    for ps, by_a in lay["runs"].items():
        header_reads(base + by_a[ps] + 8, int(ps) - 1)
    # the block ends right after the header of the last piece of run code
    assert instr.get(base + lay["end"] - 4, "").startswith("s_setpc_b64"), "end of the block is not where the table says"
    assert base + lay["end"] in instr, "no instruction at the end of the block"
    return checked


def main(asm_path, obj_path):
    lay = json.load(open(os.path.join(HERE, "ppo_pair_layout.json")))
    check_reserved_registers(open(asm_path).read(), lay)
    objdump = os.environ.get("LLVM_OBJDUMP", "/opt/rocm/llvm/bin/llvm-objdump")
    dis = subprocess.run([objdump, "-d", obj_path], check=True, capture_output=True, text=True).stdout
    n = check_entry_offsets(dis, lay)
    print(f"paired kernel: reserved registers untouched outside the blocks; {n} entry offsets verified")


if __name__ == "__main__":
    main(sys.argv[1], sys.argv[2])
