"""Helpers for scripted-rule scenarios: stacked walls and explicit action driving.

Works with any engine object offering export(), legal_mask(), step(actions) and deal_from_wall(b, wall)
(the oracle binding; the GPU binding offers the same calls).
"""
import numpy as np

from tests.handtext import tiles

J1 = "147m258p369s1234z"
J2 = "258m369p147s4567z"
J3 = "369m147p258s1235z"

A_DISCARD_RED, A_KAN, A_RIICHI, A_TSUMO, A_KYUUSHU, A_RON = 34, 37, 71, 72, 73, 74
A_PON, A_PON_RED, A_MINKAN, A_CHI_L, A_CHI_M, A_CHI_H, A_PASS = 75, 76, 77, 78, 79, 80, 84


def kind(t):
    return tiles(t)[0]


def _parse(spec):
    """'234m r5p 1z' -> list of (kind, red) ; 'r' prefix marks the red five"""
    out = []
    for tok in spec.split():
        red = tok.startswith("r")
        for k in tiles(tok[1:] if red else tok):
            out.append((k, red))
    return out


def build_wall(hands, draws="", rinshan="", dora="", ura="", dealer=0):
    """hands: 4 strings by absolute seat; draws: live draws in order (the dealer's first draw comes first)."""
    free = {k: [4 * k + c for c in range(4)] for k in range(34)}
    wall = [None] * 136

    def take(k, red):
        ids = free[k]
        if red:
            assert 4 * k in ids and k % 9 == 4 and k < 27
            ids.remove(4 * k)
            return 4 * k
        for i in reversed(ids):                      # keep copy 0 (the red one for fives) for last
            ids.remove(i)
            return i
        raise AssertionError("no copy of kind %d left" % k)

    for s in range(4):
        ts = _parse(hands[s])
        assert len(ts) == 13, (s, len(ts))
        j = (s - dealer) & 3
        for i, (k, r) in enumerate(ts):
            wall[13 * j + i] = take(k, r)
    for base, spec in ((52, draws), (122, rinshan), (126, dora), (131, ura)):
        for i, (k, r) in enumerate(_parse(spec)):
            wall[base + i] = take(k, r)
    rest = sorted(i for ids in free.values() for i in ids)
    for i in range(136):
        if wall[i] is None:
            wall[i] = rest.pop(0)
    return np.array(wall, dtype=np.uint8)


def bits(mask_row):
    return [a for a in range(85) if int(mask_row[a >> 6]) >> (a & 63) & 1]


def act(eng, b, moves):
    """Apply {seat: action} to env b (every other env gets no action); checks the actor set first."""
    e = eng.export(b, 1)[0]
    actors = {s for s in range(4) if int(e["actor_mask"]) >> s & 1}
    assert actors == set(moves), (actors, moves)
    m = eng.legal_mask()[b]
    for s, a in moves.items():
        assert a in bits(m[s]), (s, a, bits(m[s]))
    a = np.full((eng.B, 4), -1, dtype=np.int8)
    for s, x in moves.items():
        a[b, s] = x
    eng.step(a)
    return eng.export(b, 1)[0]
