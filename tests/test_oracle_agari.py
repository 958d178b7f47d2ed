"""Pins the oracle's completeness / waits functions by brute force and pattern counts."""
import ctypes as C
import itertools
import os

import numpy as np

from oracle import mjo
from tests import suitgen

SETS_ONLY, WITH_PAIR = suitgen.patterns()


def test_pattern_counts():
    by_sum = lambda d: {s: sum(1 for k in d if sum(k) == s) for s in sorted({sum(k) for k in d})}
    assert by_sum(SETS_ONLY) == {0: 1, 3: 16, 6: 127, 9: 627, 12: 2098}
    assert by_sum(WITH_PAIR) == {2: 9, 5: 135, 8: 996, 11: 4475, 14: 13259}
    assert len(SETS_ONLY) + len(WITH_PAIR) == 21743
    mult = list(SETS_ONLY.values()) + list(WITH_PAIR.values())
    assert {m: mult.count(m) for m in set(mult)} == {1: 20175, 2: 1362, 3: 190, 4: 16}
    assert sum(mult) == 23533
    assert WITH_PAIR[(0, 0, 3, 4, 4, 3, 0, 0, 0)] == 4 or SETS_ONLY.get((0, 0, 3, 4, 4, 3, 0, 0, 0), 0) == 0


def _all_vectors(max_sum=14):
    def rec(i, left, cur):
        if i == 9:
            yield tuple(cur)
            return
        for c in range(min(4, left) + 1):
            cur.append(c)
            yield from rec(i + 1, left - c, cur)
            cur.pop()
    yield from rec(0, max_sum, [])


def test_oracle_complete_on_every_single_suit_vector():
    """Every 9-count vector (entries <= 4, sum <= 14): the oracle's recursive check agrees with generation."""
    L = mjo.lib()
    buf = np.zeros(34, dtype=np.uint8)
    p = buf.ctypes.data_as(C.c_void_p)
    n = 0
    for suit in (0, 2):
        for v in _all_vectors():
            s = sum(v)
            if s % 3 == 1:
                continue
            n += 1
            buf[:] = 0
            buf[9 * suit:9 * suit + 9] = v
            if s % 3 == 2:
                if s == 14 and sorted(v) == [0, 0, 2, 2, 2, 2, 2, 2, 2]:
                    continue        # seven pairs in one suit also counts as complete; checked elsewhere
                got = L.mjo_is_complete(p, (14 - s) // 3)
                assert bool(got) == (v in WITH_PAIR), v
            else:
                if s > 12 or (s == 12 and set(v) <= {0, 2}):   # six pairs + the East pair = seven pairs
                    continue
                buf[27] = 2                                  # pair of East: the suit must be sets only
                got = L.mjo_is_complete(p, (12 - s) // 3)
                assert bool(got) == (v in SETS_ONLY), v
    assert n > 2 * 130000


def test_greedy_equals_exhaustive():
    """Triplet-first, then runs, left to right decides 'sets only' exactly (with the pair: try each pair rank)."""
    def greedy(v):
        c = list(v)
        for i in range(9):
            if c[i] >= 3:
                c[i] -= 3
            r = c[i]
            if r:
                if i > 6 or c[i + 1] < r or c[i + 2] < r:
                    return False
                c[i] = 0; c[i + 1] -= r; c[i + 2] -= r
        return True
    for v in _all_vectors():
        s = sum(v)
        if s % 3 == 0:
            assert greedy(v) == (v in SETS_ONLY), v
        elif s % 3 == 2:
            ok = False
            for p in range(9):
                if v[p] >= 2:
                    w = list(v); w[p] -= 2
                    ok = ok or greedy(w)
            assert ok == (v in WITH_PAIR), v


def _complete_by_tables(hand, n_meld):
    """completeness of a full hand from the generated per-suit sets (an independent method)"""
    if sum(hand) != 14 - 3 * n_meld:
        return False
    pairs = 0
    for s in range(3):
        v = tuple(int(x) for x in hand[9 * s:9 * s + 9])
        if v in SETS_ONLY:
            continue
        if v in WITH_PAIR:
            pairs += 1
            continue
        pairs = 99
    for k in range(27, 34):
        if hand[k] == 2:
            pairs += 1
        elif hand[k] not in (0, 3):
            pairs = 99
    std = pairs == 1
    chiitoi = n_meld == 0 and sorted(hand)[-7:] == [2] * 7 and sum(hand) == 14
    yao = [0, 8, 9, 17, 18, 26, 27, 28, 29, 30, 31, 32, 33]
    kokushi = n_meld == 0 and all(hand[k] >= 1 for k in yao) and sum(hand[k] for k in yao) == 14
    return std or chiitoi or kokushi


def _random_complete(rng, n_meld):
    while True:
        h = np.zeros(34, dtype=np.int64)
        for _ in range(4 - n_meld):
            if rng.random() < 0.5:
                k = rng.integers(34); h[k] += 3
            else:
                s, r = rng.integers(3), rng.integers(7)
                h[9 * s + r:9 * s + r + 3] += 1
        h[rng.integers(34)] += 2
        if h.max() <= 4:
            return h


def test_full_hands_against_table_method():
    rng = np.random.default_rng(1)
    n_true = 0
    for it in range(6000):
        n_meld = int(rng.integers(0, 5))
        h = _random_complete(rng, n_meld)
        if it % 2:                                   # move one tile: mostly incomplete, sometimes still complete
            src = rng.choice(np.flatnonzero(h)); h[src] -= 1
            dst = rng.choice(np.flatnonzero(h < 4)); h[dst] += 1
        want = _complete_by_tables(h.tolist(), n_meld)
        assert mjo.is_complete(h, n_meld) == want, (h, n_meld)
        n_true += want
    assert n_true > 3000
    # special forms
    chiitoi = np.zeros(34, dtype=np.uint8); chiitoi[[0, 3, 9, 13, 20, 27, 33]] = 2
    assert mjo.is_complete(chiitoi, 0) and not mjo.is_complete(chiitoi, 1)
    four = chiitoi.copy(); four[0] = 4; four[3] = 0
    assert not mjo.is_complete(four, 0)              # four of a kind is not two pairs
    koku = np.zeros(34, dtype=np.uint8); koku[[0, 8, 9, 17, 18, 26, 27, 28, 29, 30, 31, 32, 33]] = 1
    for k in (0, 17, 33):
        h = koku.copy(); h[k] += 1
        assert mjo.is_complete(h, 0)
    h = koku.copy(); h[1] += 1
    assert not mjo.is_complete(h, 0)


def test_waits_brute_force():
    rng = np.random.default_rng(2)
    seen_multi = 0
    for it in range(1500):
        n_meld = int(rng.integers(0, 4))
        h = _random_complete(rng, n_meld)
        src = rng.choice(np.flatnonzero(h)); h[src] -= 1          # a tenpai hand
        melds = []
        for j in range(n_meld):                                    # melds that do not overfill any kind
            for _ in range(50):
                k = int(rng.integers(34))
                if h[k] + 3 + sum(3 for m in melds if (m >> 3) & 63 == k) <= 4:
                    melds.append(mjo.make_meld(2, k, 1)); break
        if len(melds) != n_meld:
            continue
        w = mjo.waits_of(h, melds)
        want = 0
        for k in range(34):
            own = h[k] + sum(3 for m in melds if (m >> 3) & 63 == k)
            if own >= 4:
                continue
            h[k] += 1
            if _complete_by_tables(h.tolist(), n_meld):
                want |= 1 << k
            h[k] -= 1
        assert w == want, (h, melds)
        seen_multi += bin(w).count("1") > 1
    assert seen_multi > 200
    # the nine-sided wait of 1112345678999
    h = np.zeros(34, dtype=np.uint8); h[:9] = [3, 1, 1, 1, 1, 1, 1, 1, 3]
    assert mjo.waits_of(h) == 0x1FF
    # thirteen-sided wait
    h = np.zeros(34, dtype=np.uint8); h[[0, 8, 9, 17, 18, 26, 27, 28, 29, 30, 31, 32, 33]] = 1
    assert bin(mjo.waits_of(h)).count("1") == 13
    # a wait on a tile the player holds four of does not count: 1111m 23m... waits 1m-4m side
    h = np.zeros(34, dtype=np.uint8); h[0] = 4; h[1] = 1; h[2] = 1; h[9] = 3; h[18] = 3; h[27] = 1
    assert mjo.waits_of(h) == 1 << 27
