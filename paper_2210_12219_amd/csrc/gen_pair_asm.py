#!/usr/bin/env python3
"""Writes ppo_pair_asm.h: the register-resident row steps of the paired enumeration kernel, as inline
assembly for gfx950, and the table of entry offsets the precompute kernel needs.

A lane holds the DP row of its pair of orderings in registers: entry u (1 <= u <= 95) in v[RB + u], the lower
ordering in bits 0..15 and the upper one in bits 16..31, both as 16-bit order codes.  Output u of a row is the
minimum of the w entries u, u-1, ..., u-w+1 of the row before it (w, the window length, is the same for all
lanes and both halves: every ordering of the wave has the same node at this row) and replaces entry u in
place; the outputs are worked from the highest u down, so every input is still there when it is needed.

The code of a row is unrolled over u.  For every u there are two descending chains of packed three-input
minima (two more entries per instruction), one for even and one for odd w, that fold the entries below u into
v[RB + u] itself (its own entry always belongs to the window); a chain is entered at the step that leaves
exactly the w - 1 other entries to fold, by a computed jump whose target comes from a table the precompute
kernel wrote for this (node, row): 16-bit offsets from the block's base in units of four bytes, two per dword,
read into scalar registers.  After the last instruction of a chain a header follows (a copy of it after each
chain), which jumps to whatever the table names for the position below; a window of one entry is that header
itself.  w = 0 (no legal segment start) writes +inf.

Runs.  Consecutive outputs whose windows start at the same entry (the memory rule lets the window grow with the
segment end until a heavy layer pushes its start up) are prefix minima of one another: only the lowest output
of such a run is folded by a chain; each one above it is the minimum of the output below it and its own entry,
one instruction, `v_pk_min_u16 v[u], v[u-1], v[u]`, in ascending order.  For every end position p there is a
piece of code with these instructions for the (up to ECAP) positions ending at p, followed by a header; it is
entered at the run's second output.  Runs are worked from the top of the row down, each run from its lowest
output up; a lower run reads nothing that a higher one has written.  The table entry a header reads is the
one of the position below the code it follows; the precompute kernel (ppo_pair_program.h) fills the entries
so that the jumps walk the runs in this order and leave the block at the end.

Blocks (each one `asm volatile` statement in the kernel; fixed registers, declared clobbered there):
  LOAD     entries NE-1..1 from the lane's slot in LDS (two entries per 64-bit read, the next two ROW_BYTES on)
  LOADX    the same, then the upper half of every entry replaced by that of another slot (the pairing changes)
  ROW      entry u = max(entry u, code of t[u+s-2]/B of the lane's link), both halves the same link; then the
           chains and the run steps (one block: the row's jump table is requested while the maxima are taken)
  STORE    entries NE-1..1 to the lane's slot
  EXTRACT  entry NE-1 to an output register
  ROWMIN   the least entry of the row to an output register
Every block that works on a range of entries is entered at entry NE-1 by a computed jump (all entries of one
block have the same size).
"""
import os

HERE = os.path.dirname(os.path.abspath(__file__))

UMAX = 95            # highest entry index a row can have (L - k + 2 <= 96)
RB = 40              # entry u lives in v[RB + u]
VQ = RB + UMAX + 1   # 24 registers for the quotient dwords of the link maxima
VACC = VQ + 24       # (free)
VINF = VACC + 1
VA1 = VINF + 1       # slot address + 21 pairs of entries, + 42 pairs
VA2 = VA1 + 1
VB1 = VA2 + 1        # the same for the second slot of LOADX
VB2 = VB1 + 1
VTOP = VB2           # highest fixed register
ROW_BYTES = 384 * 8  # a slot keeps entries 2h and 2h+1 side by side (8 bytes); next pair of entries this far on
HMAX = UMAX // 2     # highest pair index
ST0 = 36             # s[ST0 .. ST0+47]: the offset table of the row (two offsets per register)
SPC = 84             # s[84:85] jump target, s[86:87] base
SBASE = 86
STMP = 88
SMASK = 89
ECAP = 16            # outputs of a run that one piece of run code takes (a longer run continues in another piece)
NSLOT = 96           # 16-bit entries of a row's table: position u reads entry (u - 1) mod 96 (position 0: the last)


def R(u):
    assert 0 <= u <= UMAX
    return f"v{RB + u}"


def RP(h):
    """the register pair of entries 2h, 2h+1 (entry 0 does not exist; its register is a dummy)"""
    return f"v[{RB + 2 * h}:{RB + 2 * h + 1}]"


def addr_for(h, a0, a1, a2):
    """address register and offset of pair h (pairs 0..20 from a0, 21..41 from a1, 42..47 from a2)."""
    if h < 21:
        return a0, h * ROW_BYTES
    if h < 42:
        return a1, (h - 21) * ROW_BYTES
    return a2, (h - 42) * ROW_BYTES


def entry_jump(stride):
    """jump to entry `skip` of the table that follows (%[skip]: entries or pairs of entries to leave out at the top)."""
    return [f"s_mul_i32 s{STMP}, %[skip], {stride}",
            f"s_add_u32 s{STMP}, s{STMP}, 12",
            f"s_getpc_b64 s[{SPC}:{SPC + 1}]",
            f"s_add_u32 s{SPC}, s{SPC}, s{STMP}",
            f"s_addc_u32 s{SPC + 1}, s{SPC + 1}, 0",
            f"s_setpc_b64 s[{SPC}:{SPC + 1}]"]


def block_load(extra):
    """extra: after the lane's own slot, the upper half of every entry is replaced by the upper half of the same
    entry of a second slot.  (A 16-bit load into a register half is no use here: on this chip it clears the other
    half.)  The second slot is read whole, 12 pairs at a time, and merged under a mask."""
    lines = [f"v_add_u32_e32 v{VA1}, {21 * ROW_BYTES}, %[addr]", f"v_add_u32_e32 v{VA2}, {42 * ROW_BYTES}, %[addr]"]
    if extra:
        lines += [f"v_add_u32_e32 v{VB1}, {21 * ROW_BYTES}, %[addr2]", f"v_add_u32_e32 v{VB2}, {42 * ROW_BYTES}, %[addr2]",
                  f"s_mov_b32 s{SMASK}, 0xffff"]
    lines += entry_jump(8)
    for h in range(HMAX, -1, -1):
        a, off = addr_for(h, "%[addr]", f"v{VA1}", f"v{VA2}")
        lines.append(f"ds_read_b64 {RP(h)}, {a} offset:{off}")
    if extra:
        for first in range(0, HMAX + 1, 12):
            hs = list(range(first, min(first + 12, HMAX + 1)))
            for n, h in enumerate(hs):
                b, off2 = addr_for(h, "%[addr2]", f"v{VB1}", f"v{VB2}")
                lines.append(f"ds_read_b64 v[{VQ + 2 * n}:{VQ + 2 * n + 1}], {b} offset:{off2}")
            lines.append("s_waitcnt lgkmcnt(0)")
            for n, h in enumerate(hs):
                for d in range(2):
                    lines.append(f"v_bfi_b32 {R(2 * h + d)}, s{SMASK}, {R(2 * h + d)}, v{VQ + 2 * n + d}")
    return lines


def block_store():
    lines = [f"v_add_u32_e32 v{VA1}, {21 * ROW_BYTES}, %[addr]", f"v_add_u32_e32 v{VA2}, {42 * ROW_BYTES}, %[addr]"]
    lines += entry_jump(8)
    for h in range(HMAX, -1, -1):
        a, off = addr_for(h, "%[addr]", f"v{VA1}", f"v{VA2}")
        lines.append(f"ds_write_b64 {a}, {RP(h)} offset:{off}")
    return lines


def block_qmax():
    """%[qaddr]: LDS byte address of the lane's quotient dword for entries 1 and 2; dword j covers entries 2j+1
    (lower half) and 2j+2 (upper half).  First the row's jump table is requested (scalar loads, used by the
    chains that follow in the same block), then the quotient dwords, 24 at a time; the second 24 are requested
    in two halves while the maxima of the first are taken, into the registers those have just freed.  The first
    wait is for everything (the loaded entries, the table: scalar loads return in any order); after it only LDS
    reads are in flight, which return in order, so the later waits count them."""
    lines = [f"s_load_dwordx16 s[{ST0}:{ST0 + 15}], %[desc], 0x0",
             f"s_load_dwordx16 s[{ST0 + 16}:{ST0 + 31}], %[desc], 0x40",
             f"s_load_dwordx16 s[{ST0 + 32}:{ST0 + 47}], %[desc], 0x80"]

    def reads(first, count):
        for j in range(first, first + count, 2):   # two dwords per read (offsets in dwords)
            lines.append(f"ds_read2_b32 v[{VQ + j % 24}:{VQ + j % 24 + 1}], %[qaddr] offset0:{j} offset1:{j + 1}")

    def maxima(first, count):
        for j in range(first, first + count):
            for h in range(2):
                u = 2 * j + 1 + h
                if u <= UMAX:
                    lines.append(f"v_pk_max_u16 {R(u)}, {R(u)}, v{VQ + j % 24} op_sel:[0,{h}] op_sel_hi:[1,{h}]")

    reads(0, 24)
    lines.append("s_waitcnt lgkmcnt(0)")
    maxima(0, 12)
    reads(24, 12)
    maxima(12, 12)
    reads(36, 12)
    lines.append("s_waitcnt lgkmcnt(6)")
    maxima(24, 12)
    lines.append("s_waitcnt lgkmcnt(0)")
    maxima(36, 12)
    return lines


def header(u):
    """what follows the code of position u + 1 (or starts the row at its highest position u): jump to the entry
    the table names for position u (0 <= u <= UMAX)."""
    slot = (u - 1) % NSLOT
    x, hi = slot // 2, slot & 1
    first = f"s_lshr_b32 s{STMP}, s{ST0 + x}, 16" if hi else f"s_and_b32 s{STMP}, s{ST0 + x}, s{SMASK}"
    return [first,
            f"s_lshl2_add_u32 s{SPC}, s{STMP}, s{SBASE}",
            f"s_addc_u32 s{SPC + 1}, s{SBASE + 1}, 0",
            f"s_setpc_b64 s[{SPC}:{SPC + 1}]"]


HEADER_BYTES = 16


def jmax_even(u):
    """three-input steps of the even chain (each folds entries u - 2i and u - 2i - 1, i = 1 ..)"""
    return max((u - 2) // 2, 0)


def jmax_odd(u):
    """three-input steps of the odd chain (each folds entries u - 2i + 1 and u - 2i)"""
    return (u - 1) // 2


def emit_first(p):
    """the lowest position the run code ending at p holds"""
    return max(2, p - ECAP + 1)


def block_compute():
    """returns (lines, offsets) with offsets[u] = (even_base, odd_base, zero), offsets['run'][p] = start of the run
    code ending at p, and offsets['end'], in bytes from the base (the instruction after s_getpc)."""
    lines = [f"s_mov_b32 s{SMASK}, 0xffff",
             f"v_mov_b32_e32 v{VINF}, 0x7c007c00",
             f"s_mul_i32 s{STMP}, %[skip], {HEADER_BYTES}",
             f"s_getpc_b64 s[{SBASE}:{SBASE + 1}]"]
    pos = 0   # bytes from the base
    body = []

    def emit(ls):
        nonlocal pos
        for ln in ls:
            body.append(ln)
            pos += size_of(ln)

    # the first header: jump to the standalone header of the highest entry (%[skip] = UMAX - highest entry here)
    emit([f"s_add_u32 s{STMP}, s{STMP}, 16",           # distance from the base to the table of standalone headers
          f"s_add_u32 s{SPC}, s{SBASE}, s{STMP}",
          f"s_addc_u32 s{SPC + 1}, s{SBASE + 1}, 0",
          f"s_setpc_b64 s[{SPC}:{SPC + 1}]"])
    assert pos == 16
    for u in range(UMAX, 0, -1):
        emit(header(u))
    assert pos == 16 + UMAX * HEADER_BYTES
    offsets = {"run": {}}
    for u in range(UMAX, 0, -1):
        nxt = header(u - 1)
        je, jo = jmax_even(u), jmax_odd(u)
        even_base = None
        if u >= 2:
            even_base = pos
            for J in range(je, 0, -1):
                emit([f"v_pk_minimum3_f16 {R(u)}, {R(u)}, {R(u - 2 * J)}, {R(u - 2 * J - 1)}"])
            emit([f"v_pk_min_u16 {R(u)}, {R(u)}, {R(u - 1)}"])
            emit(nxt)
        odd_base = pos
        for J in range(jo, 0, -1):
            emit([f"v_pk_minimum3_f16 {R(u)}, {R(u)}, {R(u - 2 * J + 1)}, {R(u - 2 * J)}"])
        emit(nxt)
        zero = pos
        emit([f"v_mov_b32_e32 {R(u)}, v{VINF}"])
        emit(nxt)
        offsets[u] = (even_base, odd_base, zero)
    for p in range(2, UMAX + 1):
        offsets["run"][p] = pos
        for x in range(emit_first(p), p + 1):
            emit([f"v_pk_min_u16 {R(x)}, {R(x - 1)}, {R(x)}"])
        emit(header(p - 1))
    offsets["end"] = pos
    return lines + body, offsets


def size_of(line):
    """bytes of one instruction of the COMPUTE block (checked against the assembled code by check_pair_code.py)"""
    op = line.split()[0]
    if op.startswith("v_pk_") or op.startswith("ds_"):
        return 8
    return 4


def block_extract():
    """%[skip] = UMAX - highest entry"""
    lines = entry_jump(8)
    for u in range(UMAX, 0, -1):
        lines += [f"v_mov_b32_e32 %[res], {R(u)}", "s_branch 1f"]
    lines.append("1:")
    return lines


def block_rowmin():
    """%[res] = the least of entries NE-1 .. 1, half by half (%[skip] = UMAX - highest entry); waits for loads first"""
    lines = ["s_waitcnt lgkmcnt(0)", "v_mov_b32_e32 %[res], 0x7c007c00"] + entry_jump(8)
    for u in range(UMAX, 0, -1):
        lines.append(f"v_pk_min_u16 %[res], %[res], {R(u)}")
    return lines


def entry_offset(offsets, u, w):
    """byte offset of the instruction at which output u with a window of w entries starts."""
    assert 0 <= w <= u
    even_base, odd_base, zero = offsets[u]
    if w == 0:
        return zero
    if w & 1:
        return odd_base + 8 * (jmax_odd(u) - (w - 1) // 2)     # (w - 1) / 2 steps, then the header
    return even_base + 8 * (jmax_even(u) - (w - 2) // 2)       # (w - 2) / 2 steps, then the two-input minimum


def run_offset(offsets, a, p):
    """byte offset at which the run code ending at p is entered so that positions a .. p are worked."""
    assert emit_first(p) <= a <= p
    return offsets["run"][p] + 8 * (a - emit_first(p))


def c_string(lines):
    return " \\\n".join('    "' + ln + '\\n"' for ln in lines)


def main():
    compute, offsets = block_compute()
    assert offsets["end"] // 4 < 65536
    clobber_v = ", ".join(f'"v{i}"' for i in range(RB, VTOP + 1))
    clobber_s = ", ".join(f'"s{i}"' for i in range(ST0, ST0 + 48)) + ", " + ", ".join(f'"s{i}"' for i in range(SPC, SMASK + 1))
    out = ["// Generated by gen_pair_asm.py; do not edit.  Row steps of the paired enumeration kernel (see the generator).",
           "#pragma once", "#include <stdint.h>", "",
           f"#define PPO_PAIR_UMAX {UMAX}",
           f"#define PPO_PAIR_HMAX {HMAX}",
           f"#define PPO_PAIR_RB {RB}",
           f"#define PPO_PAIR_VTOP {VTOP}",
           f"#define PPO_PAIR_ROW_BYTES {ROW_BYTES}",
           f"#define PPO_PAIR_CLOBBER_V {clobber_v}",
           f"#define PPO_PAIR_CLOBBER_S {clobber_s}, \"scc\"", ""]
    for name, lines in (("LOAD", block_load(False)), ("LOADX", block_load(True)), ("STORE", block_store()),
                        ("ROW", block_qmax() + compute), ("EXTRACT", block_extract()), ("ROWMIN", block_rowmin())):
        out.append(f"#define PPO_PAIR_{name}_ASM \\")
        out.append(c_string(lines))
        out.append("")
    # entry offsets for the precompute kernel, in units of four bytes from the base of COMPUTE
    ev = [0] + [(offsets[u][0] or 0) // 4 for u in range(1, UMAX + 1)]
    od = [0] + [offsets[u][1] // 4 for u in range(1, UMAX + 1)]
    ze = [0] + [offsets[u][2] // 4 for u in range(1, UMAX + 1)]
    rn = [0, 0] + [offsets["run"][p] // 4 for p in range(2, UMAX + 1)]
    out += ["#ifndef PPO_HD",
            "#ifdef __HIPCC__",
            "#define PPO_HD __host__ __device__",
            "#else",
            "#define PPO_HD",
            "#endif",
            "#endif",
            "namespace ppo {",
            f"constexpr int kPairRunCap = {ECAP};     // outputs one piece of run code takes",
            f"constexpr int kPairSlots16 = {NSLOT};   // 16-bit entries of a row's table; position u reads entry (u - 1) mod {NSLOT}",
            "// Where the pieces of the COMPUTE block start, in units of four bytes from its base: per position u the",
            "// chain for even windows, the chain for odd windows and the instruction that writes +inf; per end",
            "// position p the run code.  One constant copy; a kernel that looks offsets up many times copies it to LDS.",
            "struct PairOffsets {",
            "    uint16_t even_base[PPO_PAIR_UMAX + 1], odd_base[PPO_PAIR_UMAX + 1], zero[PPO_PAIR_UMAX + 1], run_base[PPO_PAIR_UMAX + 1];",
            "};",
            "PPO_HD inline const PairOffsets& pair_offsets() {",
            "    static constexpr PairOffsets t = {",
            "        {" + ",".join(map(str, ev)) + "},",
            "        {" + ",".join(map(str, od)) + "},",
            "        {" + ",".join(map(str, ze)) + "},",
            "        {" + ",".join(map(str, rn)) + "}};",
            "    return t;",
            "}",
            "// Where output u of a row with a window of w entries (0 <= w <= u) starts.  Even w: the even chain of u,",
            "// entered so that w / 2 - 1 steps precede its last instruction; odd w: the odd chain, (w - 1) / 2 steps",
            "// (w = 1: the header that follows it); w = 0: the instruction that writes +inf.",
            "PPO_HD inline uint32_t pair_entry_offset(const PairOffsets& t, uint32_t u, uint32_t w) {",
            "    if (w == 0u) return t.zero[u];",
            "    if (w & 1u) return t.odd_base[u] + 2u * ((u - 1u) / 2u - (w - 1u) / 2u);",
            "    return t.even_base[u] + 2u * ((u - 2u) / 2u - (w - 2u) / 2u);",
            "}",
            "// Where the run code ending at position p is entered so that the positions a .. p are worked, each the",
            "// minimum of the output below it and its own entry (2 <= a <= p, p - a < kPairRunCap).",
            "PPO_HD inline uint32_t pair_run_offset(const PairOffsets& t, uint32_t a, uint32_t p) {",
            "    const uint32_t first = p + 1u > (uint32_t)kPairRunCap + 2u ? p + 1u - (uint32_t)kPairRunCap : 2u;",
            "    return t.run_base[p] + 2u * (a - first);",
            "}",
            f"constexpr uint32_t kPairEnd = {offsets['end'] // 4};   // the end of the block",
            "}  // namespace ppo", ""]
    path = os.path.join(HERE, "ppo_pair_asm.h")
    with open(path, "w") as f:
        f.write("\n".join(out))
    # the same offsets for the build step's check of the compiled code
    import json
    with open(os.path.join(HERE, "ppo_pair_layout.json"), "w") as f:
        json.dump({"umax": UMAX, "rb": RB, "vtop": VTOP, "vacc": VACC, "vinf": VINF, "sbase": SBASE, "ecap": ECAP,
                   "nslot": NSLOT, "st0": ST0, "stmp": STMP, "smask": SMASK,
                   "entries": {str(u): {str(w): entry_offset(offsets, u, w) for w in range(0, u + 1)} for u in range(1, UMAX + 1)},
                   "runs": {str(p): {str(a): run_offset(offsets, a, p) for a in range(emit_first(p), p + 1)}
                            for p in range(2, UMAX + 1)},
                   "end": offsets["end"]}, f)
    print("wrote", path, "compute block", offsets["end"], "bytes")


if __name__ == "__main__":
    main()
