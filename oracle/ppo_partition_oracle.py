"""Oracle for the paper's partitioning step (Sec. III-B1, Alg. 1): plain Python, one instance at a time.

TEST INFRASTRUCTURE ONLY; shares no code with the library.  The step: cut the chain into segments that each fit a
node of capacity kappa (binary64 prefix sums of m, "fits" is <=) so that the sum of the transfer sizes at the
cuts is least.  Sums are binary64, added from the chain's end: cost(c_1) + (cost(c_2) + (... + 0)).
Ties: fewest segments, then the smallest first cut, second cut, ...
Two routes: `bruteforce` (every subset of cut positions, the definition) and `partition` (the recurrence over
suffixes that Alg. 1's memoised search computes).  Pins (tests/test_partition_oracle.py): closed forms and the
agreement of the two routes on integer-valued instances, where every sum is exact.
"""
import itertools
import math


def _prefix(m):
    P = [0.0]
    for x in m:
        P.append(P[-1] + float(x))
    return P


def bruteforce(t, m, kappa):
    """(segments, cuts, sum) by trying every set of cuts."""
    L = len(t)
    P = _prefix(m)
    best = None
    for p in range(1, L + 1):
        for cuts in itertools.combinations(range(1, L), p - 1):
            ends = list(cuts) + [L]
            starts = [0] + list(cuts)
            if any(not (P[e] - P[s] <= float(kappa)) for s, e in zip(starts, ends)):
                continue
            total = 0.0
            for c in reversed(cuts):
                total = float(t[c - 1]) + total
            cand = (total, p, cuts)
            if best is None or cand < best:
                best = cand
    if best is None:
        return 0, (), math.inf
    return best[1], best[2], best[0]


def partition(t, m, kappa):
    """The same by the recurrence f[i] = min over fitting e of cost(e) + f[e]."""
    L = len(t)
    P = _prefix(m)
    f = [None] * (L + 1)          # (sum, segments, first end)
    f[L] = (0.0, 0, L)
    for i in range(L - 1, -1, -1):
        best = (math.inf, 0, L)
        for e in range(i + 1, L + 1):
            if not (P[e] - P[i] <= float(kappa)):
                break
            if f[e][0] == math.inf:
                continue
            cand = ((float(t[e - 1]) if e < L else 0.0) + f[e][0], f[e][1] + 1, e)
            if cand < best:
                best = cand
        f[i] = best
    if f[0][0] == math.inf:
        return 0, (), math.inf
    cuts, e = [], f[0][2]
    while e < L:
        cuts.append(e)
        e = f[e][2]
    return f[0][1], tuple(cuts), f[0][0]
