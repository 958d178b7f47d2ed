"""Oracle phase machine: invariants over seeded random rollouts, and transition properties."""
import numpy as np
import pytest

from oracle import mjo
from tests.invariants import check_env


@pytest.mark.parametrize("flags,mode", [(mjo.RULES_NORED, mjo.MODE_SINGLE), (mjo.RULES_RED, mjo.MODE_HALF),
                                        (mjo.RULES_NORED | mjo.F_ABORT, mjo.MODE_EAST),
                                        (mjo.RULES_RED | mjo.F_ENDGAME, mjo.MODE_EAST),
                                        (mjo.RULES_RED | mjo.F_KANDORA_LATE | mjo.F_NAGASHI | mjo.F_ANKAN_ROB | mjo.F_PAO, mjo.MODE_HALF)])
def test_invariants_every_step(flags, mode):
    B = 24
    o = mjo.Oracle(B, seed=17, flags=flags, mode=mode)
    prev = o.export()
    ends = np.zeros(10, dtype=int)
    for t in range(700):
        a = o.sample_random()
        o.step(a)
        cur = o.export()
        for b in range(B):
            check_env(cur[b], flags, check_waits=(t % 7 == 0))
            _check_transition(prev[b], cur[b], a[b], flags, mode)
            if cur[b]["end_type"] and (cur[b]["kyoku_serial"] != prev[b]["kyoku_serial"] or
                                       (cur[b]["terminated"] and not prev[b]["terminated"])):
                ends[cur[b]["end_type"]] += 1
        o.reset_done()
        prev = o.export()
    assert ends[3] > 20 and ends[1] + ends[2] > 0


def _check_transition(p, c, a, flags, mode):
    """properties of one step p -> c"""
    if p["terminated"]:
        assert (c["delta"] == 0).all()
        return
    assert (c["score"] - p["score"] == c["delta"]).all()
    ended = c["kyoku_serial"] != p["kyoku_serial"] or c["terminated"]
    if not ended:
        # only a riichi stick can move points inside a kyoku
        assert set(np.unique(c["delta"])) <= {0, -1000}
        assert c["kyoku"] == p["kyoku"] and c["honba"] == p["honba"]
        return
    et = int(c["end_type"])
    dealer = int(p["kyoku"]) & 3
    if et == 9:
        return
    if et in (1, 2):
        renchan = bool(int(c["winners"]) >> dealer & 1)
        honba = int(p["honba"]) + 1 if renchan else 0
    else:
        renchan = bool(int(c["tenpai_mask"]) >> dealer & 1) if et == 3 else True
        honba = int(p["honba"]) + 1
    assert int(c["honba"]) == min(honba, 255)
    last = {0: 0, 1: 3, 2: 7}[mode]
    if not flags & mjo.F_ENDGAME:
        # the game is over after a single kyoku, when somebody is below zero, or when the last kyoku is not repeated
        over = mode == 0 or bool((c["score"] < 0).any()) or (not renchan and int(p["kyoku"]) == last)
        assert bool(c["terminated"]) == over
    if c["terminated"]:
        assert c["kyotaku"] == 0
        order = sorted(range(4), key=lambda s: (-int(c["score"][s]), s))
        assert [int(c["final_rank"][s]) for s in order] == [0, 1, 2, 3]
    else:
        assert int(c["kyoku"]) == int(p["kyoku"]) + (0 if renchan else 1)
        assert (c["score"] >= 0).all()
    if et == 3:
        T = int(c["tenpai_mask"])
        n = bin(T).count("1")
        want = np.zeros(4, dtype=np.int64)
        if 0 < n < 4:
            for s in range(4):
                want[s] = 3000 // n if T >> s & 1 else -(3000 // (4 - n))
        extra = c["delta"] - want
        if c["terminated"]:
            # the deposits left on the table go to the first in rank, and to nobody else
            top = int(np.flatnonzero(c["final_rank"] == 0)[0])
            assert extra[top] == 1000 * int(p["kyotaku"]) and extra.sum() == extra[top]
        else:
            assert (extra == 0).all()
    if et == 2:
        loser = int(c["loser"])
        assert c["delta"][loser] < 0 and not int(c["winners"]) >> loser & 1
        for s in range(4):
            if s != loser and not int(c["winners"]) >> s & 1 and not c["terminated"]:
                assert c["delta"][s] == 0
    if et == 1:
        w = int(c["winners"]).bit_length() - 1
        for s in range(4):
            if s != w:
                assert c["delta"][s] < 0


def test_modes_and_termination():
    for mode, max_kyoku in [(mjo.MODE_SINGLE, 0), (mjo.MODE_EAST, 3), (mjo.MODE_HALF, 7)]:
        o = mjo.Oracle(32, seed=5, flags=mjo.RULES_NORED, mode=mode)
        for _ in range(4000):
            o.step_random(1, auto_reset=False)
            e = o.export()
            assert e["kyoku"].max() <= max_kyoku
            if e["terminated"].all():
                break
        assert e["terminated"].all()
        if mode == mjo.MODE_SINGLE:
            assert (e["kyoku_serial"] == 0).all()
        # frozen once terminated
        before = o.export()
        o.step(np.full((32, 4), -1, dtype=np.int8))
        after = o.export()
        for n in before.dtype.names:
            if n not in ("delta", "illegal_seat"):
                assert (before[n] == after[n]).all(), n
        assert (after["delta"] == 0).all()


def test_illegal_action_terminates_with_penalty():
    o = mjo.Oracle(4, seed=1)
    m = o.legal_mask()
    a = o.sample_random()
    e0 = o.export()
    cur = int(e0["cur"][2])
    illegal = next(i for i in range(85) if not int(m[2, cur, i >> 6]) >> (i & 63) & 1)
    a[2, cur] = illegal
    a[3, int(e0["cur"][3])] = -1
    o.step(a)
    e = o.export()
    d, r, t = o.reward()
    assert t.tolist() == [0, 0, 1, 1]
    for b in (2, 3):
        c = int(e0["cur"][b])
        assert e["end_type"][b] == 9 and e["illegal_seat"][b] == c and e["phase"][b] == 3
        assert (d[b] == 0).all() and r[b, c] == -1.0 and r[b].sum() == -1.0
        assert not e["mask"][b].any()
    o.step(o.sample_random())
    d, r, t = o.reward()
    assert (r[2] == 0).all() and t.tolist() == [0, 0, 1, 1]
    o.reset_done()
    e = o.export()
    assert (e["terminated"] == 0).all() and e["episode"].tolist() == [0, 0, 1, 1] and e["kyoku_serial"].tolist() == [0, 0, 1, 1]


def test_observation_planes():
    o = mjo.Oracle(8, seed=9, flags=mjo.RULES_RED, mode=mjo.MODE_HALF)
    for _ in range(120):
        o.step_random(1)
    e, obs = o.export(), o.observe()
    assert obs.shape == (8, 4, 56, 34) and obs.max() == 1
    for b in range(8):
        for me in range(4):
            P = obs[b, me]
            assert (P[0:4].sum(0) == e["hand"][b, me]).all()                       # thermometer of own counts
            for rel in range(4):
                s = (me + rel) & 3
                riv = np.bincount(e["river"][b, s][:e["n_river"][b, s]] & 63, minlength=34)
                assert (P[5 + 4 * rel:9 + 4 * rel].sum(0) == np.minimum(riv, 4)).all()
                assert P[42 + rel].all() == bool(e["riichi"][b, s]) and P[42 + rel].any() == bool(e["riichi"][b, s])
                assert P[49 + rel].sum() == min(34, max(0, int(e["score"][b, s]) // 2000))
            assert P[46].sum() == 1 and P[46][27 + (e["kyoku"][b] >> 2)] == 1
            assert P[47].sum() == 1 and P[48].sum() == 1
            assert P[48][(int(e["kyoku"][b]) - me) & 3] == 1
            assert P[53][:18].sum() == int(e["live_left"][b]) // 4
            ind = np.bincount(e["wall"][b][126:126 + e["n_dora"][b]] >> 2, minlength=34)
            assert (P[37:41].sum(0) == ind).all()


def test_river_capacity_under_claims_that_feed_one_seat():
    """A river holds at most 32 tiles (oracle and kernels assert it).  A seat never discards more than 30 times in a
    kyoku: between two of its discards the turn goes once round the table, a live draw moves it by one seat and a
    claim by at most three, and there are at most 70 live draws and 16 claims, so 4 (n - 1) <= 70 + 48.  Here every
    seat plays to bring the turn back to seat 0 (the dealer) as often as the tiles allow: nobody wins, declares or
    makes a kan, seat 0 claims whatever it can, the seat before it claims seat 0's discards, the others claim only
    when that skips seats on the way to seat 0.  The longest river stays inside the bound (and well above the 18 to
    19 discards of a kyoku without claims, so the scenario does what it is meant to)."""
    B = 192
    o = mjo.Oracle(B, seed=3, flags=mjo.RULES_NORED, mode=mjo.MODE_SINGLE)
    longest = 0
    for _ in range(400):
        e = o.export()
        if e["terminated"].all():
            break
        m = o.legal_mask()
        a = np.full((B, 4), -1, dtype=np.int8)
        for b in range(B):
            if e["terminated"][b]:
                continue
            d = int(e["last_discarder"][b])
            for s in range(4):
                if not int(e["actor_mask"][b]) >> s & 1:
                    continue
                legal = [x for x in range(85) if int(m[b, s, x >> 6]) >> (x & 63) & 1]
                if e["phase"][b] == 0:
                    a[b, s] = [x for x in legal if x < 37][-1]          # a discard, never a declaration
                    continue
                claims = [x for x in legal if 75 <= x <= 83 and x != 77]
                # seats passed over on the way from the discarder to seat 0 if s takes the tile
                helps = s == 0 or (d == 0 and s == 3) or (s == 3 and d == 1) or (s == 2 and d == 0)
                a[b, s] = claims[0] if claims and helps else 84
        o.step(a)
        longest = max(longest, int(o.export()["n_river"].max()))
    assert 22 <= longest <= 30, longest
