"""Pins of the oracle's shanten number (paper section 3.2: a scalar of the observation).

Nothing here retypes the search: the values are tied to hand-worked examples, to the oracle's separately pinned
completeness / waits functions, and to the identities any "distance to tenpai" must satisfy."""
import os

import numpy as np
import pytest

from oracle import mjo
from tests.handtext import tiles

WALL = np.repeat(np.arange(34), 4)


def counts(kinds):
    return np.bincount(np.asarray(kinds, dtype=np.int64), minlength=34).astype(np.uint8)


def golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "shanten.txt")
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            hand, n_meld, want = line.split()[:3]
            yield hand, int(n_meld), int(want)


@pytest.mark.parametrize("hand,n_meld,want", list(golden()))
def test_worked_examples(hand, n_meld, want):
    assert mjo.shanten(counts(tiles(hand)), n_meld) == want


def _hands(rng, n, size, max_count=4, suits=None):
    wall = WALL if suits is None else np.repeat(np.concatenate([np.arange(9 * s, 9 * s + 9) for s in suits]), 4)
    out = []
    while len(out) < n:
        h = counts(rng.permutation(wall)[:size])
        if h.max() <= max_count:
            out.append(h)
    return out


def test_minus_one_means_complete_and_zero_means_tenpai():
    rng = np.random.default_rng(5)
    n_complete = n_tenpai = 0
    # hands rich in sets: two suits only, so that complete and tenpai hands actually occur
    for h in _hands(rng, 1500, 14, suits=(0,)) + _hands(rng, 1500, 14, suits=(0, 1)) + _hands(rng, 300, 14):
        done = mjo.is_complete(h, 0)
        assert (mjo.shanten(h, 0) == -1) == done
        n_complete += done
    # 13 tiles, no kind held more than three times: "tenpai" = some tile completes the hand = shanten 0
    for h in _hands(rng, 1500, 13, 3, suits=(1,)) + _hands(rng, 1500, 13, 3, suits=(0, 2)) + _hands(rng, 300, 13, 3):
        w = mjo.waits_of(h)
        assert (mjo.shanten(h, 0) == 0) == (w != 0), h.tolist()
        n_tenpai += w != 0
    # with melds: 13 - 3m concealed tiles, the melds are honor triplets that the concealed tiles avoid
    for m in (1, 2, 3):
        melds = [mjo.make_meld(2, 31 + j) for j in range(m)]
        for h in _hands(rng, 600, 13 - 3 * m, 3, suits=(0, 1)):
            assert (mjo.shanten(h, m) == 0) == (mjo.waits_of(h, melds) != 0), (h.tolist(), m)
    assert n_complete > 20 and n_tenpai > 100


def test_one_exchange_changes_the_distance_by_one():
    """what makes the number a distance: from a 13-tile hand that is s > 0 away, the best draw leads to a 14-tile
    hand that is s - 1 away (never closer), a tenpai hand has a draw that completes it, and a 14-tile hand is as far
    as its best 13-tile sub-hand.  Hands hold at most three of a kind so that every draw is possible."""
    rng = np.random.default_rng(6)
    hands = _hands(rng, 250, 13, 3) + _hands(rng, 150, 13, 3, suits=(0, 1)) + _hands(rng, 100, 13, 3, suits=(2,))
    seen = set()
    for h in hands:
        s = mjo.shanten(h, 0)
        seen.add(s)
        after_draw = []
        for t in range(34):
            g = h.copy(); g[t] += 1
            sg = mjo.shanten(g, 0)
            after_draw.append(sg)
            sub = min(mjo.shanten(g - np.eye(34, dtype=np.uint8)[d], 0) for d in np.flatnonzero(g))
            assert max(sg, 0) == sub, (g.tolist(), sg, sub)      # a complete hand's sub-hands are tenpai
        assert min(after_draw) == s - 1, (h.tolist(), s, min(after_draw))
    assert {0, 1, 2, 3, 4} <= seen


def test_bounds_and_symmetries():
    rng = np.random.default_rng(7)
    for h in _hands(rng, 500, 13):
        s = mjo.shanten(h, 0)
        assert 0 <= s <= 6                                          # seven pairs is never more than six away
        swapped = np.concatenate([h[9:18], h[0:9], h[18:]])         # exchanging two suits changes nothing
        mirrored = np.concatenate([h[0:9][::-1], h[9:]])            # nor does reversing the ranks of a suit
        assert mjo.shanten(swapped, 0) == s and mjo.shanten(mirrored, 0) == s
