#!/usr/bin/env python3
"""Writes ppo_group_tables.h: the lane/slot schedule of the grouped enumeration kernel.

The grouped kernel evaluates, in one workgroup, the 360 orderings that share a prefix of k-6 nodes
and whose arrangement of the six remaining nodes is a permutation sigma of one parity.  Each
ordering owns a DP row in LDS (a "slot").  At every row of the DP a wave works on the 60 slots
whose ordering puts the same node at that row, so that the memory window is wave-uniform.  The 60
slots of a wave must fall into distinct LDS banks per half-wave, whatever the row and node.

Construction.  Let H be the alternating group A4 acting on the six 2-subsets of {0,1,2,3}: a
subgroup of A6 of order 12, transitive on the six points with point stabilisers of order 2.  The
cosets {h o sigma : h in H} split each parity class of S6 into 30 classes of 12 permutations, and
within a class every value occurs exactly twice at every position.  Slot = (index in class, class):
rows are interleaved so that the bank of a slot is its class.  For any position r and value c the
60 permutations with sigma(r) = c are then two per class: one goes to lane `class`, the other to
lane `32 + class`, and every half-wave touches 30 distinct banks.

Tables (same for every instance):
  kLaneSlot[2][42][64]  per lane, 16 bits: bits 0..8 the slot id (index*32 + class) it handles; bits
                        9..12 the index of the unordered pair {sigma(r), sigma(r+1)} among the 15 pairs
                        of six (row-major upper triangle) for the set's position r (0 for r = 5 and for
                        the natural sets); bits 13..15 sigma(0).  Lanes 30, 31, 62, 63 are idle and
                        point at the two unused bank columns (slot ids 30 and 31), so that they never
                        collide with a working lane and need no predicate.
                        Sets 0..35 = (position r, value c) -> r*6 + c; sets 36..41 = all slots in
                        natural order (index 2n and 2n+1), used while the node is the same for all
  kSlotPerm[2][384]     per slot: sigma packed 3 bits per position, lexicographic rank of sigma
                        among the 720 permutations of six in bits 18..27, bit 31 = slot in use
                        (idle slots carry the identity permutation with bit 31 clear)
Index 0 of the first dimension holds the even permutations, index 1 the odd ones.
"""
import itertools
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def parity(p):
    inv = sum(1 for i in range(len(p)) for j in range(i + 1, len(p)) if p[i] > p[j])
    return inv & 1


def a4_on_pairs():
    pairs = list(itertools.combinations(range(4), 2))
    idx = {frozenset(p): i for i, p in enumerate(pairs)}
    H = []
    for g in itertools.permutations(range(4)):
        if parity(g) == 0:
            H.append(tuple(idx[frozenset((g[a], g[b]))] for a, b in pairs))
    assert len(set(H)) == 12 and all(parity(h) == 0 for h in H)
    return H


def build():
    H = a4_on_pairs()
    all6 = list(itertools.permutations(range(6)))
    lex = {p: i for i, p in enumerate(all6)}
    idle = [(30 + (lane & 1)) if (lane & 31) >= 30 else 0xFFFF for lane in range(64)]
    lane_slot = [[list(idle) for _ in range(42)] for _ in range(2)]
    identity = sum(v << (3 * pos) for pos, v in enumerate(range(6)))
    slot_perm = [[identity] * 384 for _ in range(2)]

    def pair6(a, b):
        lo, hi = min(a, b), max(a, b)
        return lo * 6 - lo * (lo + 1) // 2 + (hi - lo - 1)


    for par in range(2):
        perms = [p for p in all6 if parity(p) == par]
        assert len(perms) == 360
        cls_of, classes = {}, []
        for p in perms:
            if p in cls_of:
                continue
            coset = sorted({tuple(h[x] for x in p) for h in H})
            assert len(coset) == 12 and all(parity(q) == par for q in coset)
            for q in coset:
                cls_of[q] = (len(classes), coset.index(q))
            classes.append(coset)
        assert len(classes) == 30
        slot = {p: cls_of[p][1] * 32 + cls_of[p][0] for p in perms}
        for p in perms:
            packed = sum(v << (3 * pos) for pos, v in enumerate(p))
            slot_perm[par][slot[p]] = packed | (lex[p] << 18) | (1 << 31)
        for r in range(6):
            for c in range(6):
                members = sorted(p for p in perms if p[r] == c)
                assert len(members) == 60
                seen = {}
                for p in members:
                    cl = cls_of[p][0]
                    half = seen.get(cl, 0)
                    assert half < 2, "a class occurs more than twice: lanes would collide on a bank"
                    seen[cl] = half + 1
                    lane_slot[par][r * 6 + c][32 * half + cl] = slot[p]
                assert all(v == 2 for v in seen.values()) and len(seen) == 30
        for n in range(6):
            for half in range(2):
                for cl in range(30):
                    lane_slot[par][36 + n][32 * half + cl] = (2 * n + half) * 32 + cl
        # every lane set is bank-conflict free per half-wave, and the natural sets cover every slot once
        for s in range(42):
            for half in range(2):
                banks = [v & 31 for v in lane_slot[par][s][32 * half:32 * half + 32]]
                assert 0xFFFF not in lane_slot[par][s] and len(set(banks)) == 32
        covered = sorted(v for n in range(6) for l, v in enumerate(lane_slot[par][36 + n]) if (l & 31) < 30)
        assert covered == sorted(slot.values())
        perm_of = {slot[p]: p for p in perms}
        for st in range(42):
            r = st // 6 if st < 36 else None
            for lane in range(64):
                v = lane_slot[par][st][lane]
                p = perm_of.get(v, tuple(range(6)))
                link = pair6(p[r], p[r + 1]) if (r is not None and r < 5) else 0
                lane_slot[par][st][lane] = v | (link << 9) | (p[0] << 13)
    return lane_slot, slot_perm


def main():
    lane_slot, slot_perm = build()
    out = ["// Generated by gen_group_tables.py; do not edit.  Lane/slot schedule of the grouped enumeration",
           "// kernel (360 orderings per workgroup, one LDS bank per coset class).",
           "#pragma once", "#include <stdint.h>", "", "namespace ppo {", ""]
    out.append("__device__ const uint16_t kLaneSlot[2][42][64] = {")
    for par in range(2):
        out.append(" {")
        for s in range(42):
            out.append("  {" + ",".join(f"0x{v:x}" for v in lane_slot[par][s]) + "},")
        out.append(" },")
    out.append("};")
    out.append("")
    out.append("__device__ const uint32_t kSlotPerm[2][384] = {")
    for par in range(2):
        out.append(" {" + ",".join(f"0x{v:08x}u" for v in slot_perm[par]) + "},")
    out.append("};")
    out.append("")
    out.append("}  // namespace ppo")
    path = os.path.join(HERE, "ppo_group_tables.h")
    with open(path, "w") as f:
        f.write("\n".join(out) + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
