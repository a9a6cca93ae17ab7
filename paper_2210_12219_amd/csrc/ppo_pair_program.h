// The jump table of one (node, DP row) of the paired enumeration kernel: which generated code (ppo_pair_asm.h) the
// row runs through, written as the 16-bit offsets its headers read.  Plain C++ (host and device): the build step
// compiles it for the host as well and walks the tables it makes through a model of the generated code.
//
// Output u of row s (segment end e = u + s) is the minimum of the w = e - max(lo[e], s) entries u, u-1, .., u-w+1.
// Consecutive outputs whose windows start at the same entry form a run: the lowest is folded by a chain, each
// one above it is the minimum of the output below it and its own entry.  Runs are worked from the top of the row
// down, a run from its lowest output up.  The code that follows position x + 1 (or starts the row at x) reads the
// entry of position x, entry number (x - 1) mod kPairSlots16:
//   after the chain of a run's lowest output u1:   entry of u1 - 1 = the run code for u1 + 1 .. (if the run has more
//                                                  outputs), else the start of the next run below
//   after a piece of run code ending at p:         entry of p - 1  = the next piece of the same run, else the start of
//                                                  the next run below
// and the start of the run whose top is the row's highest output is the entry of that output.  Entries nothing
// reads hold the offset of the block's end, as does the one read after the last run.
#pragma once
#include <stdint.h>

#include "ppo_pair_asm.h"

namespace ppo {

PPO_HD inline int pair_slot16(int x) { return (x + kPairSlots16 - 1) % kPairSlots16; }

// lo_row: lo[j][0 .. L] of the row's node (first legal segment start per segment end); entry: kPairSlots16 offsets
PPO_HD inline void pair_row_program(int L, int k, int s, const unsigned char* lo_row, uint16_t* entry) {
    const int top = L - k + 1;   // highest output of a row
    for (int i = 0; i < kPairSlots16; ++i) entry[i] = (uint16_t)kPairEnd;
    auto window = [&](int u) -> int {
        const int e = u + s;
        const int first = (int)lo_row[e] > s ? (int)lo_row[e] : s;
        return e > first ? e - first : 0;
    };
    if (top < 1) return;
    if (s == k - 1) {   // the last row: D[L] only
        entry[pair_slot16(top)] = (uint16_t)pair_entry_offset((uint32_t)top, (uint32_t)window(top));
        return;
    }
    int pending = pair_slot16(top);   // the entry that the code worked last will read
    int u2 = top;
    while (u2 >= 1) {
        int u1 = u2;
        const int w2 = window(u2);
        if (w2 > 0) {
            const int start = u2 - w2;   // one below the lowest entry of the window: the same for the whole run
            while (u1 > 1) {
                const int wb = window(u1 - 1);
                if (wb == 0 || (u1 - 1) - wb != start) break;
                --u1;
            }
        }
        // A run of several outputs whose whole window fits one piece of run code is worked as one ascending pass
        // from the window's second entry: every entry on the way becomes the minimum of the window's entries up
        // to it.  That changes entries below the run, but only into minima of entries that any lower window
        // holding them holds as well (windows never start later than those above them), so the outputs below
        // come out the same; and it takes one jump where the chain and the run code take two.
        const int first = u2 - w2 + 1;   // lowest entry of the run's windows
        if (u2 > u1 && u2 - first <= kPairRunCap) {
            entry[pending] = (uint16_t)pair_run_offset((uint32_t)(first + 1), (uint32_t)u2);
            pending = pair_slot16(u2 - 1);
            u2 = u1 - 1;
            continue;
        }
        entry[pending] = (uint16_t)pair_entry_offset((uint32_t)u1, (uint32_t)window(u1));
        pending = pair_slot16(u1 - 1);
        for (int a = u1 + 1; a <= u2;) {
            const int p = a + kPairRunCap - 1 < u2 ? a + kPairRunCap - 1 : u2;
            entry[pending] = (uint16_t)pair_run_offset((uint32_t)a, (uint32_t)p);
            pending = pair_slot16(p - 1);
            a = p + 1;
        }
        u2 = u1 - 1;
    }
    entry[pending] = (uint16_t)kPairEnd;
}

}  // namespace ppo
