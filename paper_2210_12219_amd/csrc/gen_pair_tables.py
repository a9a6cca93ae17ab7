#!/usr/bin/env python3
"""Writes ppo_pair_tables.h: the lane schedule of the paired enumeration kernel.

A workgroup of six waves evaluates the 720 orderings that share a prefix of k-6 nodes.  A lane works on TWO
orderings at a time, one in each half of its 32-bit registers, and at every DP row a wave holds the 120
orderings (60 lanes) that put the same node at that row, so that the memory window is the same for every
lane and for both halves.

Pairs.  For the rows of the first four of the six remaining positions an ordering sigma is paired with
sigma o (4 5) (positions 4 and 5 exchanged): the two agree at positions 0..3.  For the rows of positions 4 and
5 it is paired with sigma o (0 1): they agree at positions 2..5.  Either way a pair holds exactly one even
permutation, which names the pair and sits in the lower half; the storage slot of a pair is the slot of its
even permutation.  Between the two pairings only the upper halves move.

Slots and banks.  As in the grouped kernel, the even permutations are split into the 30 cosets of a subgroup
A4 of A6 that is transitive on the six points with point stabilisers of order 2: within a coset every node
occurs exactly twice at every position.  Slot = index in coset * 32 + coset: the LDS bank of a slot is its
coset, and the 60 pairs with sigma(r) = c are two per coset, one for each half-wave.

kPairLane[6][64][4] (wave = index c of the node among the six remaining ones in ascending order; lane):
  word 0: slot at rows of positions 0, 1, 2 (9 bits each)
  word 1: slot at rows of positions 3, 4, 5
  word 2: bits 0..8 slot whose upper half holds, in the first pairing, the lane's upper ordering of position 4
          (the one that has to be fetched when the pairing changes); bits 9+4(r-1)..: index of the unordered
          pair {sigma(r-1), sigma(r)} among the 15 pairs of six, r = 1..5
  word 3: bits 0..9 rank of the lower ordering of the last row among the 720 arrangements, bits 10..19 rank
          of the upper one, bit 31 lane in use
Lanes 30, 31, 62, 63 are idle and work on spare slots (cosets 30 and 31) that no pair uses.
"""
import itertools
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def parity(p):
    return sum(1 for i in range(len(p)) for j in range(i + 1, len(p)) if p[i] > p[j]) & 1


def a4_on_pairs():
    pairs = list(itertools.combinations(range(4), 2))
    idx = {frozenset(p): i for i, p in enumerate(pairs)}
    H = []
    for g in itertools.permutations(range(4)):
        if parity(g) == 0:
            H.append(tuple(idx[frozenset((g[a], g[b]))] for a, b in pairs))
    assert len(set(H)) == 12
    return H


def swap(p, a, b):
    q = list(p)
    q[a], q[b] = q[b], q[a]
    return tuple(q)


def pair6(a, b):
    lo, hi = min(a, b), max(a, b)
    return lo * 6 - lo * (lo + 1) // 2 + (hi - lo - 1)


def build():
    H = a4_on_pairs()
    all6 = list(itertools.permutations(range(6)))
    lex = {p: i for i, p in enumerate(all6)}
    even = [p for p in all6 if parity(p) == 0]
    cls_of, classes = {}, []
    for p in even:
        if p in cls_of:
            continue
        coset = sorted({tuple(h[x] for x in p) for h in H})
        assert len(coset) == 12 and all(parity(q) == 0 for q in coset)
        for q in coset:
            cls_of[q] = (len(classes), coset.index(q))
        classes.append(coset)
    assert len(classes) == 30
    slot = {p: cls_of[p][1] * 32 + cls_of[p][0] for p in even}
    assert len(set(slot.values())) == 360 and all((s & 31) < 30 for s in slot.values())
    idle_slot = {30: 30, 31: 31, 62: 62, 63: 63}
    table = [[[0, 0, 0, 0] for _ in range(64)] for _ in range(6)]
    lane_perm = [[[None] * 6 for _ in range(64)] for _ in range(6)]
    for c in range(6):
        for r in range(6):
            members = sorted(p for p in even if p[r] == c)
            assert len(members) == 60
            seen = {}
            for p in members:
                cl = cls_of[p][0]
                half = seen.get(cl, 0)
                assert half < 2
                seen[cl] = half + 1
                lane_perm[c][32 * half + cl][r] = p
            assert len(seen) == 30 and all(v == 2 for v in seen.values())
    for c in range(6):
        for lane in range(64):
            if (lane & 31) >= 30:
                s = idle_slot[lane]
                table[c][lane] = [s | (s << 9) | (s << 18), s | (s << 9) | (s << 18), s, 0]
                continue
            ps = lane_perm[c][lane]
            slots = [slot[p] for p in ps]
            w0 = slots[0] | (slots[1] << 9) | (slots[2] << 18)
            w1 = slots[3] | (slots[4] << 9) | (slots[5] << 18)
            # the upper ordering of the row of position 4 is tau o (0 1); in the first pairing it is the upper
            # half of the pair named by (tau o (0 1)) o (4 5)
            tau = ps[4]
            partner = swap(swap(tau, 0, 1), 4, 5)
            assert parity(partner) == 0 and partner[4] != tau[4] or True
            w2 = slot[partner]
            for r in range(1, 6):
                p = ps[r]
                # both orderings of the lane's pair agree at positions r-1 and r (first pairing: r <= 3,
                # second pairing: r-1 >= 3 ... and r = 4 with r-1 = 3 >= 2)
                other = swap(p, 4, 5) if r <= 3 else swap(p, 0, 1)
                assert other[r - 1] == p[r - 1] and other[r] == p[r] and p[r] == c
                w2 |= pair6(p[r - 1], p[r]) << (9 + 4 * (r - 1))
            last = ps[5]
            w3 = lex[last] | (lex[swap(last, 0, 1)] << 10) | (1 << 31)
            table[c][lane] = [w0, w1, w2, w3]
    # checks: per (wave, row) the lanes of each half-wave hit 32 distinct banks; every pair is handled exactly once per row
    for r in range(6):
        seen = set()
        for c in range(6):
            for half in range(2):
                banks = []
                for l in range(32):
                    lane = 32 * half + l
                    w = table[c][lane]
                    s = ((w[0] >> (9 * r)) if r < 3 else (w[1] >> (9 * (r - 3)))) & 511
                    banks.append(s & 31)
                    if (lane & 31) < 30:
                        assert s not in seen
                        seen.add(s)
                assert len(set(banks)) == 32
        assert seen == set(slot.values())
    # the exchange of upper halves at position 4: every pair's upper half is fetched by exactly one lane
    fetched = sorted(table[c][lane][2] & 511 for c in range(6) for lane in range(64) if (lane & 31) < 30)
    assert fetched == sorted(slot.values())
    # the orderings of the last row cover all 720 arrangements once
    ranks = sorted(x for c in range(6) for lane in range(64) if (lane & 31) < 30
                   for x in (table[c][lane][3] & 1023, (table[c][lane][3] >> 10) & 1023))
    assert ranks == list(range(720))
    return table


def main():
    table = build()
    out = ["// Generated by gen_pair_tables.py; do not edit.  Lane schedule of the paired enumeration kernel",
           "// (720 orderings per workgroup, two per lane, one LDS bank per coset class).",
           "#pragma once", "#include <stdint.h>", "", "namespace ppo {", "",
           "__device__ const uint32_t kPairLane[6][64][4] = {"]
    for c in range(6):
        out.append(" {" + ",".join("{" + ",".join(f"0x{v:08x}u" for v in table[c][lane]) + "}" for lane in range(64)) + "},")
    out += ["};", "", "}  // namespace ppo"]
    path = os.path.join(HERE, "ppo_pair_tables.h")
    with open(path, "w") as f:
        f.write("\n".join(out) + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
