#!/usr/bin/env python3
"""Build-time checks of the paired enumeration kernel's compiled code (run by build.py; fails the build loudly).

The kernel keeps the DP row in fixed registers across several inline-assembly blocks and jumps into generated code
at offsets computed from instruction sizes.  Both rest on what the toolchain emits, so both are verified on the
code it did emit:
  1. in the compiler's assembly of the kernel, no instruction outside the blocks touches a reserved register;
  2. in the disassembly of the assembled object, the instruction at every entry offset of ppo_pair_layout.json is
     the chain or run step the table means and is followed by the steps and the header it should be (right
     chain, right depth, right registers), every header
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
    """every instantiation of the kernel; returns how many were found"""
    lo, hi = lay["rb"], lay["vtop"]   # entry 0 has a (dummy) register too
    inside_kernel = in_asm = False
    kernels = seen_blocks = 0
    for n, line in enumerate(asm_text.splitlines(), 1):
        if re.match(rf"^_ZN3ppo\d+{KERNEL}\w*:", line):
            inside_kernel = True
            kernels += 1
            seen_blocks = 0
            continue
        if not inside_kernel:
            continue
        if line.startswith(".Lfunc_end"):
            assert seen_blocks >= 5, "the kernel's blocks were not found in the assembly"
            inside_kernel = False
            continue
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
    assert kernels >= 1 and not inside_kernel, "kernel not found in the assembly"
    return kernels


def kernel_listings(disasm_text):
    """instructions by address, one dict per instantiation of the kernel"""
    out, instr = [], None
    for line in disasm_text.splitlines():
        if re.match(rf"^[0-9a-f]+ <_ZN3ppo\d+{KERNEL}\w*>:", line):
            instr = {}
            out.append(instr)
            continue
        if instr is not None and re.match(r"^[0-9a-f]+ <", line):
            instr = None
            continue
        if instr is not None:
            m = re.match(r"^\s*(\S.*?)\s*//\s*([0-9A-Fa-f]+):", line)
            if m:
                instr[int(m.group(2), 16)] = re.sub(r"\s+", " ", m.group(1).strip())
    return out


def check_entry_offsets(instr, lay):
    sb = lay["sbase"]
    bases = [a for a, t in instr.items() if t == f"s_getpc_b64 s[{sb}:{sb + 1}]"]
    assert len(bases) == 1, f"expected one base instruction, found {len(bases)}"
    base = bases[0] + 4
    rb, vinf = lay["rb"], lay["vinf"]
    st0, nslot = lay["st0"], lay["nslot"]
    R = lambda u: f"v{rb + u}"

    def header_text(position):
        """first instruction of a header that reads the table entry of `position`"""
        slot = (position - 1) % nslot
        x, hi = slot // 2, slot & 1
        return (f"s_lshr_b32 s{lay['stmp']}, s{st0 + x}, 16" if hi
                else f"s_and_b32 s{lay['stmp']}, s{st0 + x}, s{lay['smask']}")

    def expect(addr, want, what):
        got = instr.get(addr)
        assert got == want, f"{what} at +{addr - base}: found `{got}`, expected `{want}`"

    checked = 0
    for us, by_w in lay["entries"].items():
        u = int(us)
        for ws, off in by_w.items():
            w = int(ws)
            what = f"entry u={u} w={w}"
            if w == 0:
                expect(base + off, f"v_mov_b32_e32 {R(u)}, v{vinf}", what)
                expect(base + off + 4, header_text(u - 1), what + " (header)")
            elif w & 1:
                J = (w - 1) // 2      # steps to run; then the header of the position below
                for i in range(J, 0, -1):
                    expect(base + off + 8 * (J - i), f"v_pk_minimum3_f16 {R(u)}, {R(u)}, {R(u - 2 * i + 1)}, {R(u - 2 * i)}", what)
                expect(base + off + 8 * J, header_text(u - 1), what + " (header)")
            else:
                J = (w - 2) // 2
                for i in range(J, 0, -1):
                    expect(base + off + 8 * (J - i), f"v_pk_minimum3_f16 {R(u)}, {R(u)}, {R(u - 2 * i)}, {R(u - 2 * i - 1)}", what)
                expect(base + off + 8 * J, f"v_pk_min_u16 {R(u)}, {R(u)}, {R(u - 1)}", what)
                expect(base + off + 8 * J + 8, header_text(u - 1), what + " (header)")
            checked += 1
    # the run code: entered at position a of the piece ending at p, one instruction per position up to p, each the
    # minimum of the output below and the position's own entry; then the header of position p - 1
    for ps, by_a in lay["runs"].items():
        p = int(ps)
        for as_, off in by_a.items():
            a = int(as_)
            expect(base + off, f"v_pk_min_u16 {R(a)}, {R(a - 1)}, {R(a)}", f"run code p={p} a={a}")
            checked += 1
        expect(base + by_a[ps] + 8, header_text(p - 1), f"run code p={p} (header)")
    # the block ends right after the header of the last piece of run code
    assert instr.get(base + lay["end"] - 4, "").startswith("s_setpc_b64"), "end of the block is not where the table says"
    assert base + lay["end"] in instr, "no instruction at the end of the block"
    return checked


def main(asm_path, obj_path):
    lay = json.load(open(os.path.join(HERE, "ppo_pair_layout.json")))
    kernels = check_reserved_registers(open(asm_path).read(), lay)
    objdump = os.environ.get("LLVM_OBJDUMP", "/opt/rocm/llvm/bin/llvm-objdump")
    dis = subprocess.run([objdump, "-d", obj_path], check=True, capture_output=True, text=True).stdout
    listings = kernel_listings(dis)
    assert len(listings) == kernels, f"{kernels} kernels in the assembly, {len(listings)} in the object"
    n = sum(check_entry_offsets(instr, lay) for instr in listings)
    print(f"paired kernel ({kernels} instantiations): reserved registers untouched outside the blocks; {n} entry offsets verified")


if __name__ == "__main__":
    main(sys.argv[1], sys.argv[2])
