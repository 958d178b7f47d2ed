"""Seeded generator of the hand-evaluation micro-batch.

Half of the hands are 14 tiles drawn uniformly from a shuffled 136-tile wall (almost never complete); half are
constructed complete hands: four random sets (run or triplet), 0..3 of them exposed as chi / pon / concealed kan /
open kan, plus a pair, with a winning tile drawn from the concealed tiles, a tsumo / ron coin, uniform winds and
1..4 dora indicators.  Records use the 64-byte query layout of the library (the dtype is passed in, so this
module depends on neither implementation).
"""
import numpy as np


def _random_draws(rng, n, q):
    keys = rng.random((n, 136), dtype=np.float32)
    ids = np.argsort(keys, axis=1)[:, :14]
    kinds = ids >> 2
    hand = np.zeros((n, 34), dtype=np.uint8)
    np.add.at(hand, (np.repeat(np.arange(n), 14), kinds.reshape(-1)), 1)
    q["hand"] = hand
    q["n_meld"] = 0
    q["win_kind"] = kinds[np.arange(n), rng.integers(0, 14, n)]


def _constructed(rng, n, q):
    hand = np.zeros((n, 34), dtype=np.int16)
    total = np.zeros((n, 34), dtype=np.int16)
    meld = np.zeros((n, 4), dtype=np.uint16)
    n_meld = np.zeros(n, dtype=np.uint8)
    todo = np.arange(n)
    while todo.size:
        m = todo.size
        h = np.zeros((m, 34), dtype=np.int16)
        t = np.zeros((m, 34), dtype=np.int16)
        ml = np.zeros((m, 4), dtype=np.uint16)
        n_exp = rng.integers(0, 4, m)
        rows = np.arange(m)
        for j in range(4):
            is_run = rng.random(m) < 0.5
            suit, start = rng.integers(0, 3, m), rng.integers(0, 7, m)
            k_run = 9 * suit + start
            k_tri = rng.integers(0, 34, m)
            exposed = j < n_exp
            kan = rng.integers(0, 3, m)                     # triplet exposed as: 0 pon, 1 concealed kan, 2 open kan
            for d in range(3):
                np.add.at(t, (rows[is_run], k_run[is_run] + d), 1)
                np.add.at(h, (rows[is_run & ~exposed], k_run[is_run & ~exposed] + d), 1)
            tri = ~is_run
            np.add.at(t, (rows[tri], k_tri[tri]), 3)
            np.add.at(t, (rows[tri & exposed & (kan > 0)], k_tri[tri & exposed & (kan > 0)]), 1)
            np.add.at(h, (rows[tri & ~exposed], k_tri[tri & ~exposed]), 3)
            mtype = np.where(is_run, 1, np.where(kan == 0, 2, np.where(kan == 1, 4, 3)))
            kind = np.where(is_run, k_run, k_tri)
            word = mtype | kind << 3 | rng.integers(1, 4, m) << 9 | np.where(is_run, rng.integers(0, 3, m), 0) << 11
            ml[:, j] = np.where(exposed, word, 0)
        pair = rng.integers(0, 34, m)
        np.add.at(t, (rows, pair), 2)
        np.add.at(h, (rows, pair), 2)
        ok = t.max(axis=1) <= 4
        good = todo[ok]
        hand[good], total[good], meld[good], n_meld[good] = h[ok], t[ok], ml[ok], n_exp[ok]
        todo = todo[~ok]
    # winning tile: uniform over the concealed tiles
    csum = np.cumsum(hand, axis=1)
    pick = (rng.random(n) * csum[:, -1]).astype(np.int64)
    q["win_kind"] = (csum > pick[:, None]).argmax(axis=1)
    q["hand"] = hand.astype(np.uint8)
    q["meld"] = meld
    q["n_meld"] = n_meld


def generate(n, dtype, seed=0):
    """n query records (numpy structured array of `dtype`), first half random draws, second half constructed"""
    rng = np.random.Generator(np.random.PCG64(seed))
    q = np.zeros(n, dtype=dtype)
    half = n // 2
    for lo in range(0, half, 65536):
        hi = min(half, lo + 65536)
        _random_draws(rng, hi - lo, q[lo:hi])
    for lo in range(half, n, 65536):
        hi = min(n, lo + 65536)
        _constructed(rng, hi - lo, q[lo:hi])
    tsumo = rng.random(n) < 0.5
    flags = tsumo.astype(np.uint8)
    flags |= (rng.random(n) < 0.3).astype(np.uint8) << 1       # ippatsu
    flags |= (rng.random(n) < 0.05).astype(np.uint8) << 2      # rinshan
    flags |= (rng.random(n) < 0.05).astype(np.uint8) << 3      # chankan
    flags |= (rng.random(n) < 0.05).astype(np.uint8) << 4      # haitei
    flags |= (rng.random(n) < 0.05).astype(np.uint8) << 5      # houtei
    flags |= (rng.random(n) < 0.02).astype(np.uint8) << 6      # first turn
    q["flags"] = flags
    q["riichi"] = np.where(rng.random(n) < 0.5, 0, rng.integers(1, 3, n))
    q["seat_wind"] = rng.integers(0, 4, n)
    q["round_wind"] = rng.integers(0, 2, n)
    q["n_ind"] = rng.integers(1, 5, n)
    q["ind"] = rng.integers(0, 34, (n, 5))
    q["ura"] = rng.integers(0, 34, (n, 5))
    q["n_aka"] = np.where(rng.random(n) < 0.7, 0, rng.integers(1, 3, n))
    q["kuitan"] = 1
    return q
