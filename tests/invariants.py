"""State invariants that hold after every step, for exported env records of either implementation."""
import numpy as np

from oracle import mjo      # only the plain completeness function is used, as the independent recompute


def meld_count(m, k):
    t, b = m & 7, (m >> 3) & 63
    if t == 1:
        return 1 if b <= k <= b + 2 else 0
    if t == 2:
        return 3 if k == b else 0
    if t in (3, 4, 5):
        return 4 if k == b else 0
    return 0


def check_env(e, flags, start_score=25000, check_waits=True):
    red_rules = bool(flags & 1)
    # 136 tiles conserved: per kind 4, per red five 1
    cnt = np.zeros(34, dtype=np.int64)
    reds = np.zeros(3, dtype=np.int64)
    undrawn = list(range(int(e["draw_ptr"]), 122)) + list(range(122 + int(e["n_kan"]), 136))
    for i in undrawn:
        t = int(e["wall"][i])
        cnt[t >> 2] += 1
        if red_rules and t in (16, 52, 88):
            reds[(t >> 2) // 9] += 1
    for s in range(4):
        cnt += e["hand"][s]
        for su in range(3):
            if e["hand_red"][s] >> su & 1:
                assert e["hand"][s][9 * su + 4] >= 1
                reds[su] += 1
        for j in range(int(e["n_meld"][s])):
            m = int(e["meld"][s][j])
            for k in range(34):
                cnt[k] += meld_count(m, k)
            if m >> 13 & 1:
                reds[((m >> 3) & 63) // 9] += 1
        for j in range(int(e["n_meld"][s]), 4):
            assert e["meld"][s][j] == 0
        n = int(e["n_river"][s])
        assert n <= 32
        assert (e["river"][s][n:] == 0).all()
        for i in range(n):
            t = int(e["river"][s][i])
            if not t >> 7:
                cnt[t & 63] += 1
                if t >> 6 & 1:
                    reds[(t & 63) // 9] += 1
    assert (cnt == 4).all(), cnt
    assert (reds == (1 if red_rules else 0)).all(), reds
    # points conserved
    assert int(e["score"].sum()) + 1000 * int(e["kyotaku"]) == 4 * start_score
    assert int(e["live_left"]) == 70 - (int(e["draw_ptr"]) - 52) - int(e["n_kan"])
    assert int(e["n_dora"]) + int(e["dora_pending"]) == 1 + int(e["n_kan"]) and int(e["n_kan"]) == int(e["kan_by"].sum())
    assert int(e["dora_pending"]) <= (1 if flags & 32 else 0)       # only an open or added kan defers its indicator
    # masks
    am = int(e["actor_mask"])
    if e["terminated"]:
        assert e["phase"] == 3 and am == 0 and not e["mask"].any()
    else:
        assert e["phase"] in (0, 1, 2) and am != 0
        for s in range(4):
            has = bool(e["mask"][s].any())
            assert has == bool(am >> s & 1)
            assert int(e["mask"][s][1]) >> 21 == 0          # only 85 action bits
        if e["phase"] == 0:
            assert am == 1 << int(e["cur"])
        else:
            other = int(e["last_discarder"]) if e["phase"] == 1 else int(e["cur"])
            assert not am >> other & 1
            for s in range(4):
                if am >> s & 1:
                    assert int(e["mask"][s][1]) >> (84 - 64) & 1     # PASS always offered
    # hand sizes, riichi implies closed hand, waits cache
    for s in range(4):
        n_meld = int(e["n_meld"][s])
        want = 13 - 3 * n_meld
        if not e["terminated"] and e["phase"] == 0 and s == e["cur"]:
            want += 1
        if not e["terminated"]:
            assert int(e["hand"][s].sum()) == want, (s, e["hand"][s].sum(), want)
        if e["riichi"][s]:
            assert all(int(e["meld"][s][j]) & 7 == 4 for j in range(n_meld))
        if check_waits and int(e["hand"][s].sum()) == 13 - 3 * n_meld:
            w = mjo.waits_of(e["hand"][s], [int(x) for x in e["meld"][s][:n_meld]])
            assert w == int(e["waits"][s]), (s, hex(w), hex(int(e["waits"][s])))
