"""Independent generator of decomposable single-suit patterns.

Builds every multiset of j sets (7 runs + 9 triplets) plus an optional pair and keeps those whose nine
counts stay <= 4.  This is generation, not testing: it shares no logic with the oracle's recursive checker
nor with the GPU table builder.
"""
import itertools
from collections import defaultdict

SETS = [tuple(1 if r <= i <= r + 2 else 0 for i in range(9)) for r in range(7)] + \
       [tuple(3 if i == r else 0 for i in range(9)) for r in range(9)]


def patterns():
    """-> (sets_only, with_pair): dict key(tuple of 9 counts) -> number of distinct decompositions"""
    sets_only, with_pair = defaultdict(int), defaultdict(int)
    for j in range(5):
        for combo in itertools.combinations_with_replacement(range(16), j):
            c = [0] * 9
            for s in combo:
                for i in range(9):
                    c[i] += SETS[s][i]
            if max(c) <= 4:
                sets_only[tuple(c)] += 1
            for p in range(9):
                c[p] += 2
                if max(c) <= 4:
                    with_pair[tuple(c)] += 1
                c[p] -= 2
    return dict(sets_only), dict(with_pair)
