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

// window length of output u of row s; lo_row: lo[j][0 .. L] of the row's node (first legal segment start per end)
PPO_HD inline int pair_window(int s, const unsigned char* lo_row, int u) {
    const int e = u + s;
    const int first = (int)lo_row[e] > s ? (int)lo_row[e] : s;
    return e > first ? e - first : 0;
}
// What the program of a row is made from: below[u] = u - w(u), the position just below output u's window
// (kPairNoWindow if the window is empty), for u = 1 .. top.  Outputs with equal `below` next to each other form a run.
constexpr unsigned char kPairNoWindow = 0xFF;
PPO_HD inline unsigned char pair_below(int s, const unsigned char* lo_row, int u) {
    const int w = pair_window(s, lo_row, u);
    return w > 0 ? (unsigned char)(u - w) : kPairNoWindow;
}
// the highest output of the run whose lowest output is u1
PPO_HD inline int pair_run_top(const unsigned char* below, int top, int u1) {
    int u2 = u1;
    const unsigned char b = below[u1];
    if (b != kPairNoWindow)
        while (u2 < top && below[u2 + 1] == b) ++u2;
    return u2;
}

// The entries that position u of a row is responsible for: none unless u is the lowest output of a run; else the
// entry that leads to the run (the row's first jump for the top run, otherwise the one the run above leaves to
// be read) and the entries read within the run.  Every entry has one writer, so the positions can be worked in
// any order or side by side, on entries preset to the offset of the block's end.  below: see pair_below,
// indexed by position (index 0 unused); last_row: only the highest output is wanted (D[L]).
PPO_HD inline void pair_row_program_at(const PairOffsets& t, int top, bool last_row, const unsigned char* below, int u,
                                       uint16_t* entry) {
    if (u < 1 || u > top) return;
    const int w = below[u] == kPairNoWindow ? 0 : u - (int)below[u];
    if (last_row) {
        if (u == top) entry[pair_slot16(top)] = (uint16_t)pair_entry_offset(t, (uint32_t)top, (uint32_t)w);
        return;
    }
    if (u > 1 && w > 0 && below[u - 1] == below[u]) return;   // the output below belongs to the same run
    const int u2 = pair_run_top(below, top, u);
    int pending;   // the entry that the code worked before this run reads
    if (u2 == top) {
        pending = pair_slot16(top);
    } else {
        const int a1 = u2 + 1;
        const int a2 = pair_run_top(below, top, a1);
        pending = a2 > a1 ? pair_slot16(a2 - 1) : pair_slot16(a1 - 1);
    }
    // A run of several outputs whose whole window fits one piece of run code is worked as one ascending pass
    // from the window's second entry: every entry on the way becomes the minimum of the window's entries up
    // to it.  That changes entries below the run, but only into minima of entries that any lower window
    // holding them holds as well (windows never start later than those above them), so the outputs below
    // come out the same; and it takes one jump where the chain and the run code take two.
    const int first = u - w + 1;   // lowest entry of the run's windows
    if (u2 > u && u2 - first <= kPairRunCap) {
        entry[pending] = (uint16_t)pair_run_offset(t, (uint32_t)(first + 1), (uint32_t)u2);
        pending = pair_slot16(u2 - 1);
    } else {
        entry[pending] = (uint16_t)pair_entry_offset(t, (uint32_t)u, (uint32_t)w);
        pending = pair_slot16(u - 1);
        for (int a = u + 1; a <= u2;) {
            const int p = a + kPairRunCap - 1 < u2 ? a + kPairRunCap - 1 : u2;
            entry[pending] = (uint16_t)pair_run_offset(t, (uint32_t)a, (uint32_t)p);
            pending = pair_slot16(p - 1);
            a = p + 1;
        }
    }
    if (u == 1) entry[pending] = (uint16_t)kPairEnd;   // after the lowest run the block is left
}

// entry: kPairSlots16 offsets
PPO_HD inline void pair_row_program(int L, int k, int s, const unsigned char* lo_row, uint16_t* entry) {
    const int top = L - k + 1;   // highest output of a row
    unsigned char below[PPO_PAIR_UMAX + 2];
    for (int u = 1; u <= top && u <= PPO_PAIR_UMAX; ++u) below[u] = pair_below(s, lo_row, u);
    for (int i = 0; i < kPairSlots16; ++i) entry[i] = (uint16_t)kPairEnd;
    for (int u = 1; u <= top; ++u) pair_row_program_at(pair_offsets(), top, s == k - 1, below, u, entry);
}

}  // namespace ppo
