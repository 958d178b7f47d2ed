"""Both observation formats pinned by hand on one scripted kyoku (paper section 3.2, "Observation Space").

The kyoku (red rules, East-2: seat 1 deals, two counters, one deposit, unequal points) holds a concealed kan, a
riichi whose declaration tile is claimed, a pon that uses the red five from the hand, a chi from the previous seat,
a red five thrown into a river, a red kan-dora indicator, two equal indicators, a tile added to the pon, the offer to
rob it and the replacement draw.  Every expected plane and every expected token field below was written out by hand
from the layout's definition, viewer by viewer (seats turned to the viewer by hand too); nothing is computed from an
engine.  Runs on the oracle, on the host build of the kernels' code, and (marked gpu) on the HIP library.
"""
import numpy as np
import pytest

from oracle import mjo
from tests.engines import make_engine
from tests.handtext import tiles
from tests.scenario import (A_CHI_H, A_CHI_M, A_KAN, A_PASS, A_PON, A_PON_RED, A_RIICHI, A_RON, act, bits, build_wall,
                            kind)

ALL = "ALL"
HANDS = ["239m 27p 128s 2367z 7z",               # seat 0 (north)
         "58m 234678p 99s 111z",                 # seat 1 (east, dealer)
         "46m r5p 888p 234567s 2z",              # seat 2 (south)
         "1m r5m 5m 19p 39s 34z 55z 67z"]        # seat 3 (west)


@pytest.fixture(params=["oracle", "hostsim", pytest.param("gpu", marks=pytest.mark.gpu)])
def eng(request):
    o = make_engine(request.param, 1, seed=0, flags=mjo.RULES_RED, mode=mjo.MODE_HALF)
    e = o.export()
    e["kyoku"], e["honba"], e["kyotaku"] = 1, 2, 1
    e["score"][0] = [31000, 18000, 27000, 23000]
    o.import_(e)
    o.deal_from_wall(0, build_wall(HANDS, draws="1z 4z 2z 5m", rinshan="9m 6z", dora="3p r5s 3p", dealer=1))
    yield o
    o.close()


def plane(spec):
    """hand-typed row of a plane: tile text -> those kinds set; int n -> entries 0..n-1 set; list -> those entries;
    ALL -> all 34"""
    row = np.zeros(34, dtype=np.uint8)
    if isinstance(spec, str) and spec == ALL:
        row[:] = 1
    elif isinstance(spec, str):
        row[tiles(spec.replace(" ", ""))] = 1
    elif isinstance(spec, int):
        row[:spec] = 1
    else:
        row[list(spec)] = 1
    return row


def check_planes(o, want_by_viewer, planes=range(56)):
    obs = o.observe()[0]
    assert obs.shape == (4, 56, 34)
    for me, want in enumerate(want_by_viewer):
        for p in planes:
            exp = plane(want.get(p, ""))
            assert np.array_equal(obs[me, p], exp), "viewer %d plane %d: %s, expected %s" % (
                me, p, np.flatnonzero(obs[me, p]).tolist(), np.flatnonzero(exp).tolist())


def check_tokens(o, want_by_viewer):
    t = o.observe_tokens()[0]
    for me, want in enumerate(want_by_viewer):
        for name, exp in want.items():
            got = np.asarray(t[name][me])
            if name in ("hand", "dora"):
                exp = list(exp) + [255] * (got.shape[0] - len(exp))
            elif name == "river":
                exp = [list(r) + [255] * (32 - len(r)) for r in exp]
            elif name == "meld":
                exp = [list(m) + [0] * (4 - len(m)) for m in exp]
            elif name == "hist":
                exp = list(exp) + [0xFFFF] * (128 - len(exp))
            assert got.tolist() == exp, "viewer %d field %s: %s, expected %s" % (
                me, name, got.tolist(), exp)
        assert (np.asarray(t["zero_"][me]) == 0).all()


def mk(*parts):
    out = {}
    for d in parts:
        out.update(d)
    return out


# bits of plane 53: wall tiles left in fours, counters, deposits
def scalars(live_fours, honba, kyotaku):
    return list(range(live_fours)) + [18 + i for i in range(honba)] + [26 + i for i in range(kyotaku)]


# meld words, typed from the format type | kind << 3 | from_rel << 9 | called_pos << 11 | has_red << 13 | called_red << 14
ANKAN_1Z = 4 + (27 << 3)                                   # 220
PON_5M = 2 + (4 << 3) + (2 << 9) + (1 << 13)               # 9250: from the seat across, holds the red five
KAKAN_5M = 5 + (4 << 3) + (2 << 9) + (1 << 13)             # 9253
CHI_123S = 1 + (18 << 3) + (3 << 9) + (2 << 11)            # 5777: from the previous seat, the called tile is the high one
CALLED = 0x80


def test_scripted_kyoku_planes_and_tokens(eng):
    o = eng
    # seat 1 draws the fourth east: concealed kan, the second indicator (the red 5s) is turned, replacement tile 9m
    e = act(o, 0, {1: A_KAN + kind("1z")})
    assert e["n_dora"] == 2 and e["drawn"] == kind("9m") and e["live_left"] == 68
    e = act(o, 0, {1: A_RIICHI})
    assert bits(e["mask"][1]) == [kind("5m")]
    e = act(o, 0, {1: kind("5m")})
    # ---- A: the declaration tile waits for answers: seat 2 may chi, seat 3 may pon with its red five
    assert e["phase"] == 1 and bits(e["mask"][2]) == [A_CHI_M, A_PASS] and bits(e["mask"][3]) == [A_PON_RED, A_PASS]
    hand0 = {0: "239m 27p 128s 2367z", 1: "7z"}
    scores_a = [15, 9, 13, 11]                               # 31000, 18000, 27000, 23000 in steps of 2000
    base_a = {37: "3p5s", 41: "5s", 46: "1z", 53: scalars(17, 2, 1), 54: "5m"}
    A = [mk(base_a, hand0, {9: "5m", 25: "1z", 26: "1z", 27: "1z", 28: "1z", 47: "4z", 48: [1],
                                  49: scores_a[0], 50: scores_a[1], 51: scores_a[2], 52: scores_a[3]}),
         mk(base_a, {0: "89m 234678p 9s", 1: "9s", 5: "5m", 21: "1z", 22: "1z", 23: "1z", 24: "1z", 47: "1z", 48: [0],
                         49: scores_a[1], 50: scores_a[2], 51: scores_a[3], 52: scores_a[0]}),
         mk(base_a, {0: "46m 58p 234567s 2z", 1: "8p", 2: "8p", 4: "5p", 17: "5m",
                         33: "1z", 34: "1z", 35: "1z", 36: "1z", 47: "2z", 48: [3],
                         49: scores_a[2], 50: scores_a[3], 51: scores_a[0], 52: scores_a[1]}),
         mk(base_a, {0: "15m 19p 39s 34567z", 1: "5m5z", 4: "5m", 13: "5m",
                         29: "1z", 30: "1z", 31: "1z", 32: "1z", 47: "3z", 48: [2],
                         49: scores_a[3], 50: scores_a[0], 51: scores_a[1], 52: scores_a[2]})]
    check_planes(o, A)
    check_tokens(o, [
        dict(phase=1, cur=255, drawn=255, last_discarder=1, last_discard=4, dealer=1, kyotaku=1, riichi=[0, 0, 0, 0],
             river=[[], [4], [], []], riichi_idx=[255] * 4, score=[31000, 18000, 27000, 23000]),
        dict(phase=1, cur=255, drawn=255, last_discarder=0, last_discard=4, dealer=0, river=[[4], [], [], []],
             hand=[7, 8, 10, 11, 12, 14, 15, 16, 26, 26], n_hand=10, shanten=0),
        dict(phase=1, cur=255, drawn=255, last_discarder=3, last_discard=4, dealer=3, river=[[], [], [], [4]],
             hand=[3, 5, 35, 16, 16, 16, 19, 20, 21, 22, 23, 24, 28], n_hand=13),
        dict(phase=1, cur=255, drawn=255, last_discarder=2, last_discard=4, dealer=2, river=[[], [], [4], []],
             hand=[0, 34, 4, 9, 17, 20, 26, 29, 30, 31, 31, 32, 33], n_hand=13, dora=[11, 36], n_dora=2)])

    # the pon wins over the chi; the riichi stands (1000 paid); seat 3 throws 3s, seat 0 takes it with 1s2s
    e = act(o, 0, {2: A_CHI_M, 3: A_PON_RED})
    assert e["cur"] == 3 and e["score"].tolist() == [31000, 17000, 27000, 23000] and e["meld"][3][0] == PON_5M
    e = act(o, 0, {3: kind("3s")})
    assert bits(e["mask"][0]) == [A_CHI_H, A_PASS]
    e = act(o, 0, {0: A_CHI_H})
    assert e["meld"][0][0] == CHI_123S and kind("3s") not in bits(e["mask"][0])
    e = act(o, 0, {0: kind("7z")})
    # ---- B: seat 1, in riichi, has drawn the north
    assert e["phase"] == 0 and e["cur"] == 1 and bits(e["mask"][1]) == [kind("4z")]
    sc = [15, 8, 13, 11]                                     # 31000, 17000, 27000, 23000
    base = {37: "3p5s", 41: "5m5s", 46: "1z", 53: scalars(16, 2, 2)}
    B = [mk(base, {0: "239m 27p 8s 2367z", 5: "7z", 9: "5m", 17: "3s", 21: "123s",
                       25: "1z", 26: "1z", 27: "1z", 28: "1z", 33: "5m", 34: "5m", 35: "5m", 43: ALL,
                       47: "4z", 48: [1], 49: sc[0], 50: sc[1], 51: sc[2], 52: sc[3]}),
         mk(base, {0: "89m 234678p 9s 4z", 1: "9s", 5: "5m", 13: "3s", 17: "7z",
                       21: "1z", 22: "1z", 23: "1z", 24: "1z", 29: "5m", 30: "5m", 31: "5m", 33: "123s", 42: ALL,
                       47: "1z", 48: [0], 49: sc[1], 50: sc[2], 51: sc[3], 52: sc[0], 55: "4z"}),
         mk(base, {0: "46m 58p 234567s 2z", 1: "8p", 2: "8p", 4: "5p", 9: "3s", 13: "7z", 17: "5m",
                       25: "5m", 26: "5m", 27: "5m", 29: "123s", 33: "1z", 34: "1z", 35: "1z", 36: "1z", 45: ALL,
                       47: "2z", 48: [3], 49: sc[2], 50: sc[3], 51: sc[0], 52: sc[1]}),
         mk(base, {0: "1m 19p 9s 34567z", 1: "5z", 5: "3s", 9: "7z", 13: "5m",
                       21: "5m", 22: "5m", 23: "5m", 25: "123s", 29: "1z", 30: "1z", 31: "1z", 32: "1z", 44: ALL,
                       47: "3z", 48: [2], 49: sc[3], 50: sc[0], 51: sc[1], 52: sc[2]})]
    check_planes(o, B)
    hist_b = [(1, A_KAN + 27), (1, A_RIICHI), (1, 4), (3, A_PON_RED), (3, 20), (0, A_CHI_H), (0, 33)]
    check_tokens(o, [
        dict(hand=[1, 2, 8, 10, 15, 25, 28, 29, 32, 33], n_hand=10, shanten=5, drawn=255, phase=0, cur=1,
             last_discarder=0, last_discard=33, kyoku=1, honba=2, kyotaku=2, dealer=1, live_left=67, n_dora=2,
             dora=[11, 36], n_meld=[1, 1, 0, 1], n_river=[1, 1, 0, 1], riichi=[0, 1, 0, 0], riichi_idx=[255, 0, 255, 255],
             score=[31000, 17000, 27000, 23000], meld=[[CHI_123S], [ANKAN_1Z], [], [PON_5M]],
             river=[[33], [4 | CALLED], [], [20 | CALLED]], n_hist=7,
             hist=[64 | 1 << 8, 71 | 1 << 8, 4 | 1 << 8, 76 | 3 << 8, 20 | 3 << 8, 80, 33]),
        dict(hand=[7, 8, 10, 11, 12, 14, 15, 16, 26, 26, 30], n_hand=11, shanten=0, drawn=30, phase=0, cur=0,
             last_discarder=3, last_discard=33, dealer=0, n_meld=[1, 0, 1, 1], n_river=[1, 0, 1, 1],
             riichi=[1, 0, 0, 0], riichi_idx=[0, 255, 255, 255], score=[17000, 27000, 23000, 31000],
             meld=[[ANKAN_1Z], [], [PON_5M], [CHI_123S]], river=[[4 | CALLED], [], [20 | CALLED], [33]], n_hist=7,
             hist=[64, 71, 4, 76 | 2 << 8, 20 | 2 << 8, 80 | 3 << 8, 33 | 3 << 8]),
        dict(hand=[3, 5, 35, 16, 16, 16, 19, 20, 21, 22, 23, 24, 28], n_hand=13, drawn=255, phase=0, cur=3,
             last_discarder=2, last_discard=33, dealer=3, n_meld=[0, 1, 1, 1], n_river=[0, 1, 1, 1],
             riichi=[0, 0, 0, 1], riichi_idx=[255, 255, 255, 0], score=[27000, 23000, 31000, 17000],
             meld=[[], [PON_5M], [CHI_123S], [ANKAN_1Z]], river=[[], [20 | CALLED], [33], [4 | CALLED]], n_hist=7,
             hist=[64 | 3 << 8, 71 | 3 << 8, 4 | 3 << 8, 76 | 1 << 8, 20 | 1 << 8, 80 | 2 << 8, 33 | 2 << 8]),
        dict(hand=[0, 9, 17, 26, 29, 30, 31, 31, 32, 33], n_hand=10, drawn=255, phase=0, cur=2,
             last_discarder=1, last_discard=33, dealer=2, n_meld=[1, 1, 1, 0], n_river=[1, 1, 1, 0],
             riichi=[0, 0, 1, 0], riichi_idx=[255, 255, 0, 255], score=[23000, 31000, 17000, 27000],
             meld=[[PON_5M], [CHI_123S], [ANKAN_1Z], []], river=[[20 | CALLED], [33], [4 | CALLED], []], n_hist=7,
             hist=[64 | 2 << 8, 71 | 2 << 8, 4 | 2 << 8, 76, 20, 80 | 1 << 8, 33 | 1 << 8])])
    assert [(w >> 8, w & 255) for w in e["hist"][:7].tolist()] == hist_b

    # seat 1 throws the north, seat 2 draws a south and throws its red 5p, seat 3 draws the last 5m and adds it to the pon
    e = act(o, 0, {1: kind("4z")})
    assert e["cur"] == 2 and A_RIICHI in bits(e["mask"][2])
    e = act(o, 0, {2: 35})
    assert e["cur"] == 3 and e["drawn"] == kind("5m")
    e = act(o, 0, {3: A_KAN + kind("5m")})
    # ---- C: seat 2 waits on the 5m between its 4m and 6m and may rob the kan
    assert e["phase"] == 2 and e["actor_mask"] == 0b0100 and bits(e["mask"][2]) == [A_RON, A_PASS] and e["n_dora"] == 2
    base = {37: "3p5s", 41: "5m5p5s", 46: "1z", 53: scalars(16, 2, 2), 54: "5m"}
    C = [mk(base, {0: "239m 27p 8s 2367z", 5: "7z", 9: "5m4z", 13: "5p", 17: "3s", 21: "123s",
                       25: "1z", 26: "1z", 27: "1z", 28: "1z", 33: "5m", 34: "5m", 35: "5m", 36: "5m", 43: ALL,
                       47: "4z", 48: [1], 49: sc[0], 50: sc[1], 51: sc[2], 52: sc[3]}),
         mk(base, {0: "89m 234678p 9s", 1: "9s", 5: "5m4z", 9: "5p", 13: "3s", 17: "7z",
                       21: "1z", 22: "1z", 23: "1z", 24: "1z", 29: "5m", 30: "5m", 31: "5m", 32: "5m", 33: "123s", 42: ALL,
                       47: "1z", 48: [0], 49: sc[1], 50: sc[2], 51: sc[3], 52: sc[0]}),
         mk(base, {0: "46m 8p 234567s 2z", 1: "8p2z", 2: "8p", 5: "5p", 9: "3s", 13: "7z", 17: "5m4z",
                       25: "5m", 26: "5m", 27: "5m", 28: "5m", 29: "123s", 33: "1z", 34: "1z", 35: "1z", 36: "1z", 45: ALL,
                       47: "2z", 48: [3], 49: sc[2], 50: sc[3], 51: sc[0], 52: sc[1]}),
         mk(base, {0: "1m 19p 9s 34567z", 1: "5z", 5: "3s", 9: "7z", 13: "5m4z", 17: "5p",
                       21: "5m", 22: "5m", 23: "5m", 24: "5m", 25: "123s", 29: "1z", 30: "1z", 31: "1z", 32: "1z", 44: ALL,
                       47: "3z", 48: [2], 49: sc[3], 50: sc[0], 51: sc[1], 52: sc[2]})]
    check_planes(o, C)
    check_tokens(o, [
        dict(phase=2, cur=255, drawn=255, last_discarder=2, last_discard=35, live_left=65, n_hist=10,
             meld=[[CHI_123S], [ANKAN_1Z], [], [KAKAN_5M]], river=[[33], [4 | CALLED, 30], [35], [20 | CALLED]]),
        dict(phase=2, cur=255, drawn=255, last_discarder=1, last_discard=35, hand=[7, 8, 10, 11, 12, 14, 15, 16, 26, 26]),
        dict(phase=2, cur=255, drawn=255, last_discarder=0, last_discard=35, shanten=0, n_hand=13,
             hand=[3, 5, 16, 16, 16, 19, 20, 21, 22, 23, 24, 28, 28], river=[[35], [20 | CALLED], [33], [4 | CALLED, 30]]),
        dict(phase=2, cur=255, drawn=255, last_discarder=3, last_discard=35, n_hand=10,
             hand=[0, 9, 17, 26, 29, 30, 31, 31, 32, 33], meld=[[KAKAN_5M], [CHI_123S], [ANKAN_1Z], []])])

    # seat 2 lets it go: the third indicator (a second 3p) is turned, seat 3 takes the replacement tile (green)
    e = act(o, 0, {2: A_PASS})
    # ---- D
    assert e["phase"] == 0 and e["cur"] == 3 and e["n_dora"] == 3 and e["furiten_temp"][2] == 1 and e["live_left"] == 64
    for want in C:
        want[38] = "3p"
        del want[54]
    C[3][1] = "56z"
    C[3][55] = "6z"
    check_planes(o, C)
    hist_d = [(1, 64), (1, 71), (1, 4), (3, 76), (3, 20), (0, 80), (0, 33), (1, 30), (2, 35), (3, 41)]
    assert [(w >> 8, w & 255) for w in e["hist"][:10].tolist()] == hist_d and e["n_hist"] == 10
    check_tokens(o, [
        dict(hand=[1, 2, 8, 10, 15, 25, 28, 29, 32, 33], n_hand=10, shanten=5, drawn=255, phase=0, cur=3,
             last_discarder=2, last_discard=35, kyoku=1, honba=2, kyotaku=2, dealer=1, live_left=64, n_dora=3,
             dora=[11, 36, 11], n_meld=[1, 1, 0, 1], n_river=[1, 2, 1, 1], riichi=[0, 1, 0, 0],
             riichi_idx=[255, 0, 255, 255], score=[31000, 17000, 27000, 23000],
             meld=[[CHI_123S], [ANKAN_1Z], [], [KAKAN_5M]], river=[[33], [4 | CALLED, 30], [35], [20 | CALLED]], n_hist=10,
             hist=[64 | 1 << 8, 71 | 1 << 8, 4 | 1 << 8, 76 | 3 << 8, 20 | 3 << 8, 80, 33, 30 | 1 << 8, 35 | 2 << 8,
                   41 | 3 << 8]),
        dict(hand=[7, 8, 10, 11, 12, 14, 15, 16, 26, 26], n_hand=10, shanten=0, drawn=255, phase=0, cur=2,
             last_discarder=1, last_discard=35, dealer=0, dora=[11, 36, 11], n_meld=[1, 0, 1, 1], n_river=[2, 1, 1, 1],
             riichi=[1, 0, 0, 0], riichi_idx=[0, 255, 255, 255], score=[17000, 27000, 23000, 31000],
             meld=[[ANKAN_1Z], [], [KAKAN_5M], [CHI_123S]], river=[[4 | CALLED, 30], [35], [20 | CALLED], [33]], n_hist=10,
             hist=[64, 71, 4, 76 | 2 << 8, 20 | 2 << 8, 80 | 3 << 8, 33 | 3 << 8, 30, 35 | 1 << 8, 41 | 2 << 8]),
        dict(hand=[3, 5, 16, 16, 16, 19, 20, 21, 22, 23, 24, 28, 28], n_hand=13, shanten=0, drawn=255, phase=0, cur=1,
             last_discarder=0, last_discard=35, dealer=3, dora=[11, 36, 11], n_meld=[0, 1, 1, 1], n_river=[1, 1, 1, 2],
             riichi=[0, 0, 0, 1], riichi_idx=[255, 255, 255, 0], score=[27000, 23000, 31000, 17000],
             meld=[[], [KAKAN_5M], [CHI_123S], [ANKAN_1Z]], river=[[35], [20 | CALLED], [33], [4 | CALLED, 30]], n_hist=10,
             hist=[64 | 3 << 8, 71 | 3 << 8, 4 | 3 << 8, 76 | 1 << 8, 20 | 1 << 8, 80 | 2 << 8, 33 | 2 << 8, 30 | 3 << 8,
                   35, 41 | 1 << 8]),
        dict(hand=[0, 9, 17, 26, 29, 30, 31, 31, 32, 32, 33], n_hand=11, shanten=4, drawn=32, phase=0, cur=0,
             last_discarder=3, last_discard=35, dealer=2, dora=[11, 36, 11], n_meld=[1, 1, 1, 0], n_river=[1, 1, 2, 1],
             riichi=[0, 0, 1, 0], riichi_idx=[255, 255, 0, 255], score=[23000, 31000, 17000, 27000],
             meld=[[KAKAN_5M], [CHI_123S], [ANKAN_1Z], []], river=[[20 | CALLED], [33], [4 | CALLED, 30], [35]], n_hist=10,
             hist=[64 | 2 << 8, 71 | 2 << 8, 4 | 2 << 8, 76, 20, 80 | 1 << 8, 33 | 1 << 8, 30 | 2 << 8, 35 | 3 << 8, 41])])


def test_red_five_inside_a_chi_and_claimed_from_a_river(request):
    """the red five taken from the hand into a run that starts below it (the visible-reds plane marks the five, not
    the run's lowest tile), and a red five thrown and claimed for a pon (red and claimed bits of the river entry,
    both red bits of the meld word)"""
    for which in ("oracle", "hostsim"):
        _red_chi(make_engine(which, 1, seed=0, flags=mjo.RULES_RED, mode=mjo.MODE_SINGLE))


@pytest.mark.gpu
def test_red_five_inside_a_chi_and_claimed_from_a_river_gpu():
    _red_chi(make_engine("gpu", 1, seed=0, flags=mjo.RULES_RED, mode=mjo.MODE_SINGLE))


def _red_chi(o):
    hands = ["3p 147m 28p 369s 1234z", "4p r5p r5m 28m 39p 147s 567z", "258m 369p 147s 4567z", "55m 39m 147p 258s 135z"]
    o.deal_from_wall(0, build_wall(hands, draws="9m", dora="1s"))
    e = act(o, 0, {0: kind("3p")})
    assert bits(e["mask"][1]) == [81, A_PASS]                 # only the run with the red five: no plain 5p in the hand
    e = act(o, 0, {1: 81})
    chi = 1 + (11 << 3) + (3 << 9) + (0 << 11) + (1 << 13)    # 9817: 3p4p5p, claimed low tile from the previous seat, red inside
    assert e["meld"][1][0] == chi and e["hand_red"][1] == 1
    e = act(o, 0, {1: 34})                                    # throws the red 5m
    assert bits(e["mask"][3]) == [A_PON, A_PASS]
    e = act(o, 0, {3: A_PON})
    pon = 2 + (4 << 3) + (2 << 9) + (1 << 13) + (1 << 14)     # 25634: from the seat across, the claimed tile is the red one
    assert e["meld"][3][0] == pon and e["river"][1][0] == 4 + 64 + 128 and e["hand_red"].tolist() == [0, 0, 0, 0]
    base = {41: "5m5p"}
    want = [mk(base, {5: "3p", 9: "5m", 25: "345p", 33: "5m", 34: "5m", 35: "5m"}),
            mk(base, {5: "5m", 17: "3p", 21: "345p", 29: "5m", 30: "5m", 31: "5m"}),
            mk(base, {13: "3p", 17: "5m", 25: "5m", 26: "5m", 27: "5m", 33: "345p"}),
            mk(base, {9: "3p", 13: "5m", 21: "5m", 22: "5m", 23: "5m", 29: "345p"})]
    check_planes(o, want, planes=[4] + list(range(5, 37)) + [41, 54, 55])
    check_tokens(o, [
        dict(meld=[[], [chi], [], [pon]], river=[[11 | CALLED], [34 | CALLED], [], []], last_discard=34, last_discarder=1),
        dict(meld=[[chi], [], [pon], []], river=[[34 | CALLED], [], [], [11 | CALLED]], last_discard=34, last_discarder=0),
        dict(meld=[[], [pon], [], [chi]], river=[[], [], [11 | CALLED], [34 | CALLED]], last_discard=34, last_discarder=3),
        dict(meld=[[pon], [], [chi], []], river=[[], [11 | CALLED], [34 | CALLED], []], last_discard=34, last_discarder=2,
             cur=0, drawn=255)])
    o.close()
