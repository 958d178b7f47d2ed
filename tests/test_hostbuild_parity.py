"""CPU tier: the code of the HIP kernels, compiled for the host (tests/hostsim), against the oracle.

This is the same per-environment source every kernel runs (one lane per environment); running it here lets
the GPU-less tier catch logic differences before a GPU is involved.  The GPU parity proper is test_gpu_*.py.
"""
import numpy as np
import pytest

from oracle import mjo
from tests.engines import diff_records
from tests.hostsim.sim import HostSim
from workloads import hands


def test_table_counts():
    keys, recs, rows = HostSim(1).table_stats()
    assert (keys, recs) == (21743, 23533) and rows == 98        # 97 distinct rows + the empty one


def test_hand_microbatch():
    q = hands.generate(1 << 15, mjo.QUERY_DTYPE, seed=3)
    ro, rh = mjo.eval_hands(q), HostSim(1).eval_hands(q)
    assert ro.tobytes() == rh.tobytes()
    assert ro["yaku_ok"].sum() > 5000


@pytest.mark.parametrize("flags,mode,steps", [(mjo.RULES_NORED, mjo.MODE_SINGLE, 160), (mjo.RULES_RED, mjo.MODE_HALF, 1200),
                                              (mjo.RULES_NORED | mjo.F_ABORT, mjo.MODE_EAST, 500),
                                              (mjo.RULES_RED | mjo.F_ENDGAME, mjo.MODE_EAST, 900),
                                              (mjo.RULES_RED | mjo.F_KANDORA_LATE | mjo.F_NAGASHI | mjo.F_ANKAN_ROB | mjo.F_PAO, mjo.MODE_HALF, 900)])
def test_rollout_trace(flags, mode, steps):
    B = 48
    o, s = mjo.Oracle(B, 7, flags, mode), HostSim(B, 7, flags, mode)
    for t in range(steps):
        d = diff_records(o.export(), s.export())
        assert not d, (t, d[:4])
        a, a2 = o.sample_random(), s.sample_random()
        assert np.array_equal(a, a2), t
        o.step(a); s.step(a)
        if t % 3 == 0:
            o.reset_done(); s.reset_done()
    assert np.array_equal(o.observe(), s.observe())


def test_fused_rollout_and_waits():
    o, s = mjo.Oracle(32, 1, mjo.RULES_RED, mjo.MODE_HALF), HostSim(32, 1, mjo.RULES_RED, mjo.MODE_HALF)
    o.step_random(700); s.step_random(700)
    eo, es = o.export(), s.export()
    assert not diff_records(eo, es)
    for b in range(32):
        for seat in range(4):
            n = int(eo["n_meld"][b, seat])
            if int(eo["hand"][b, seat].sum()) == 13 - 3 * n:
                assert s.waits_of(eo["hand"][b, seat], eo["meld"][b, seat][:n].tolist()) == int(eo["waits"][b, seat])


def _near_hands(rng, n):
    """Seeded 14 - 3m tile hands that sit close to tenpai in every way the waits code distinguishes: complete
    standard hands with 0-2 tiles swapped, one-suit hands, seven-pairs and thirteen-orphans neighbours, plain
    random draws; 0-3 melds (chi, pon, open / concealed / added kan)."""
    yao = [0, 8, 9, 17, 18, 26, 27, 28, 29, 30, 31, 32, 33]
    out = []
    while len(out) < n:
        left = np.full(34, 4, dtype=np.int64)
        hand = np.zeros(34, dtype=np.int64)
        melds = []
        style = int(rng.integers(0, 6))
        m = int(rng.integers(0, 4)) if style < 3 else 0
        ok = True
        for _ in range(m):
            t = int(rng.integers(1, 6))
            if t == 1:
                su, lo = int(rng.integers(0, 3)), int(rng.integers(0, 7))
                ks = [9 * su + lo + i for i in range(3)]
                if min(left[ks]) < 1: ok = False; break
                left[ks] -= 1
                melds.append(1 | ks[0] << 3 | 3 << 9)
            else:
                k, need = int(rng.integers(0, 34)), 3 if t == 2 else 4
                if left[k] < need: ok = False; break
                left[k] -= need
                melds.append(t | k << 3 | (0 if t == 4 else 2 << 9))
        if not ok:
            continue
        size = 14 - 3 * m

        def take(k):
            if left[k] < 1: return False
            left[k] -= 1; hand[k] += 1
            return True
        if style in (0, 1):                       # sets + pair, then a few tiles swapped
            one_suit = style == 1 and m == 0
            su0 = int(rng.integers(0, 3))
            for _ in range(4 - m):
                if rng.integers(0, 2) or one_suit:
                    su, lo = (su0 if one_suit else int(rng.integers(0, 3))), int(rng.integers(0, 7))
                    ks = [9 * su + lo + i for i in range(3)]
                else:
                    ks = [int(rng.integers(0, 34))] * 3
                ok = ok and all(take(k) for k in ks)
            kp = 9 * su0 + int(rng.integers(0, 9)) if one_suit else int(rng.integers(0, 34))
            ok = ok and take(kp) and take(kp)
            if not ok:
                continue
            for _ in range(int(rng.integers(0, 3))):
                held = np.flatnonzero(hand)
                d = int(rng.choice(held)); hand[d] -= 1; left[d] += 1
                a = 9 * su0 + int(rng.integers(0, 9)) if one_suit else int(rng.integers(0, 34))
                if not take(a): hand[d] += 1; left[d] -= 1
        elif style == 2:                          # plain random draw
            wall = np.repeat(np.arange(34), left)
            for k in rng.permutation(wall)[:size]: hand[k] += 1
        elif style == 3:                          # seven pairs and neighbours
            ks = rng.permutation(34)[:7]
            for k in ks: hand[k] += 2
            for _ in range(int(rng.integers(0, 3))):
                d = int(rng.choice(np.flatnonzero(hand))); a = int(rng.integers(0, 34))
                if hand[a] < 4: hand[d] -= 1; hand[a] += 1
        elif style == 4:                          # thirteen orphans and neighbours
            for k in yao: hand[k] += 1
            hand[int(rng.choice(yao))] += 1
            for _ in range(int(rng.integers(0, 3))):
                d = int(rng.choice(np.flatnonzero(hand)))
                a = int(rng.choice(yao)) if rng.integers(0, 3) else int(rng.integers(0, 34))
                if hand[a] < 4: hand[d] -= 1; hand[a] += 1
        else:                                     # 14 tiles of one suit
            su = int(rng.integers(0, 3))
            wall = np.repeat(np.arange(9 * su, 9 * su + 9), 4)
            for k in rng.permutation(wall)[:14]: hand[k] += 1
        if hand.sum() == size and hand.max() <= 4:
            out.append((hand.astype(np.uint8), melds))
    return out


def test_waits_and_tenpai_discards_vs_oracle():
    s = HostSim(1, 0, mjo.RULES_NORED, mjo.MODE_SINGLE)
    rng = np.random.default_rng(20577)
    n_tenpai = n_wait = 0
    for hand, melds in _near_hands(rng, 6000):
        want = 0
        for d in np.flatnonzero(hand):
            g = hand.copy(); g[d] -= 1
            w = mjo.waits_of(g, melds)
            assert s.waits_of(g, melds) == w, (hand.tolist(), melds, int(d))
            n_wait += w != 0
            if w: want |= 1 << int(d)
        assert s.tenpai_discards_of(hand, melds) == want, (hand.tolist(), melds)
        n_tenpai += want != 0
    assert n_tenpai > 1500 and n_wait > 5000        # the cases are not vacuous


def test_shanten_tables_vs_oracle():
    """the kernels' table-driven shanten number against the oracle's exhaustive search: random hands of every size,
    one- and two-suit hands (where the per-suit statistics are stressed), the seeded near-tenpai hands"""
    s = HostSim(1, 0, mjo.RULES_NORED, mjo.MODE_SINGLE)
    rng = np.random.default_rng(99)
    wall = np.repeat(np.arange(34), 4)
    seen = set()
    for m in (0, 1, 2, 3, 4):
        for size in (13 - 3 * m, 14 - 3 * m):
            for suits in (None, (0,), (1, 2), (2, 3)):
                w = wall if suits is None else np.repeat(np.concatenate([np.arange(9 * u, 9 * u + (7 if u == 3 else 9)) for u in suits]), 4)
                for _ in range(150):
                    h = np.bincount(rng.permutation(w)[:size], minlength=34).astype(np.uint8)
                    want = mjo.shanten(h, m)
                    assert s.shanten(h, m) == want, (h.tolist(), m)
                    seen.add(want)
    for hand, melds in _near_hands(rng, 1500):
        assert s.shanten(hand, len(melds)) == mjo.shanten(hand, len(melds)), (hand.tolist(), len(melds))
    assert set(range(-1, 7)) <= seen


def test_token_observation_trace():
    o, s = mjo.Oracle(24, 3, mjo.RULES_RED, mjo.MODE_HALF), HostSim(24, 3, mjo.RULES_RED, mjo.MODE_HALF)
    for _ in range(40):
        o.step_random(13); s.step_random(13)
        a, b = o.observe_tokens(), s.observe_tokens()
        for name in a.dtype.names:
            assert np.array_equal(a[name], b[name]), name
