"""Scripted scenarios, one rule each, on stacked walls.  Expected values follow from the rule text.

Every scenario runs on the oracle, on the host build of the kernels' code, and (marked gpu) on the HIP library.
"""
import numpy as np
import pytest

from oracle import mjo
from tests.engines import make_engine
from tests.scenario import (A_CHI_H, A_CHI_L, A_CHI_M, A_KAN, A_PASS, A_PON, A_RIICHI, A_RON, A_TSUMO, A_KYUUSHU,
                            A_MINKAN, J1, J2, J3, act, bits, build_wall, kind)
from tests.invariants import check_env

TENPAI = "234m 34p 456p 22s 678s"          # waits 2p / 5p; pinfu + tanyao
TENPAI2 = "234m 34p 678p 33s 678s"         # the same waits from different tiles


@pytest.fixture(params=["oracle", "hostsim", pytest.param("gpu", marks=pytest.mark.gpu)])
def engine(request):
    def make(flags=mjo.RULES_NORED, mode=mjo.MODE_SINGLE, **kw):
        return make_engine(request.param, 1, seed=0, flags=flags, mode=mode, **kw)
    return make


def test_tenhou(engine):
    o = engine()
    o.deal_from_wall(0, build_wall([TENPAI, J1, J2, J3], draws="5p", dora="1z"))
    e = o.export()[0]
    assert bits(e["mask"][0]).count(A_TSUMO) == 1 and A_RIICHI in bits(e["mask"][0])
    e = act(o, 0, {0: A_TSUMO})
    assert e["end_type"] == 1 and e["winners"] == 1 and e["yakuman_units"][0] == 1 and e["yaku"][0] == 1 << 42
    assert e["delta"].tolist() == [48000, -16000, -16000, -16000] and e["terminated"] == 1
    assert e["final_rank"].tolist() == [0, 1, 2, 3] and e["gain"][0] == 48000


def test_double_ron_honba_sticks_and_rotation(engine):
    o = engine(mode=mjo.MODE_HALF)
    o.deal_from_wall(0, build_wall(["5p " + J1[1:], TENPAI, TENPAI2, J3], draws="1m", dora="1z"))
    e = o.export()
    e["honba"], e["kyotaku"] = 2, 1
    e["score"][0] = [25000, 25000, 25000, 24000]
    o.import_(e)
    e = act(o, 0, {0: kind("5p")})
    assert e["phase"] == 1 and e["actor_mask"] == 0b0110
    assert bits(e["mask"][1]) == [A_RON, A_CHI_M, A_CHI_H, A_PASS]       # next seat may also chi with 4p6p / 3p4p
    assert bits(e["mask"][2]) == [A_RON, A_PASS]
    e = act(o, 0, {1: A_RON, 2: A_RON})
    assert e["end_type"] == 2 and e["winners"] == 0b0110 and e["loser"] == 0
    assert e["han"].tolist() == [0, 2, 2, 0] and e["fu"].tolist() == [0, 30, 30, 0]
    # 2000 + 2 honba * 300 each; the stick goes to seat 1, the first after the loser
    assert e["delta"].tolist() == [-5200, 3600, 2600, 0] and e["gain"].tolist() == [0, 3600, 2600, 0]
    assert e["kyoku"] == 1 and e["honba"] == 0 and e["kyotaku"] == 0 and e["kyoku_serial"] == 1
    assert e["cur"] == 1 and e["phase"] == 0 and e["terminated"] == 0       # next kyoku dealt in the same step
    check_env(e, mjo.RULES_NORED)


def test_pon_beats_chi_and_kuikae(engine):
    o = engine()
    hands = [J1, "4567m258p369s567z", "44m 369p147s456z 11p", J3]
    o.deal_from_wall(0, build_wall(hands, draws="1m"))
    e = act(o, 0, {0: kind("4m")})
    assert e["actor_mask"] == 0b0110
    assert bits(e["mask"][1]) == [A_CHI_L, A_PASS] and bits(e["mask"][2]) == [A_PON, A_PASS]
    e = act(o, 0, {1: A_CHI_L, 2: A_PON})
    assert e["cur"] == 2 and e["phase"] == 0 and e["n_meld"].tolist() == [0, 0, 1, 0]
    m = int(e["meld"][2][0])
    assert m & 7 == 2 and (m >> 3) & 63 == kind("4m") and (m >> 9) & 3 == 2       # pon, taken from the seat across
    assert e["river"][0][0] == kind("4m") | 0x80 and e["drawn"] == 255
    legal = bits(e["mask"][2])
    assert kind("4m") not in legal and A_TSUMO not in legal and all(a < 34 for a in legal)
    assert (e["first_turn"] == 0).all()
    # now the chi alone: forbidden are the called kind and the kind three above it
    o.deal_from_wall(0, build_wall([J1, hands[1], J2, J3], draws="1m"))
    e = act(o, 0, {0: kind("4m")})
    assert e["actor_mask"] == 0b0010
    e = act(o, 0, {1: A_CHI_L})
    m = int(e["meld"][1][0])
    assert m & 7 == 1 and (m >> 3) & 63 == kind("4m") and (m >> 9) & 3 == 3 and (m >> 11) & 3 == 0
    legal = bits(e["mask"][1])
    assert kind("4m") not in legal and kind("7m") not in legal and kind("2p") in legal
    assert e["kuikae"].tolist() == [kind("4m"), kind("7m")]
    e = act(o, 0, {1: kind("2p")})
    assert e["kuikae"].tolist() == [255, 255] and e["cur"] == 2


def test_furiten_permanent_and_temporary(engine):
    # own discard among the waits: no ron
    o = engine()
    o.deal_from_wall(0, build_wall(["5p " + J1[1:], TENPAI, J2, J3], draws="1m"))
    e = o.export()
    e["discarded_kinds"][0][1] = 1 << kind("2p")
    o.import_(e)
    e = act(o, 0, {0: kind("5p")})
    assert A_RON not in bits(e["mask"][1]) and e["furiten_temp"][1] == 1
    # passing a ron: furiten until the own next discard
    o = engine()
    hands = ["5p " + J1[1:], TENPAI, "2p 58m369p147s4567z", J3]
    o.deal_from_wall(0, build_wall(hands, draws="1m 9m 9m 9s 1s"))
    e = act(o, 0, {0: kind("5p")})
    assert A_RON in bits(e["mask"][1])
    e = act(o, 0, {1: A_PASS})
    assert e["furiten_temp"][1] == 1 and e["cur"] == 1
    e = act(o, 0, {1: kind("9m")})
    assert e["furiten_temp"][1] == 0
    e = act(o, 0, {2: kind("9m")})                       # seat 2 cuts its draw; nobody can call it
    e = act(o, 0, {3: kind("9s")})
    e = act(o, 0, {0: kind("2p")})
    assert A_RON in bits(e["mask"][1])                     # the temporary furiten is over


def test_temporary_furiten_blocks_same_go_around(engine):
    o = engine()
    hands = ["5p " + J1[1:], J3, "2p 58m369p147s4567z", TENPAI]
    # seat 3 waits on 2p/5p; seat 0 cuts 5p (seat 3 passes), then seat 2 cuts 2p in the same go-around
    o.deal_from_wall(0, build_wall(hands, draws="1m 9m 9m"))
    e = act(o, 0, {0: kind("5p")})
    assert e["actor_mask"] == 0b1000
    e = act(o, 0, {3: A_PASS})
    assert e["furiten_temp"][3] == 1
    e = act(o, 0, {1: kind("9m")})
    e = act(o, 0, {2: kind("2p")})
    assert bits(e["mask"][3]) == [A_CHI_L, A_PASS]               # the shape fits, but no ron in the same go-around


def test_riichi_ippatsu_tsumo_ura(engine):
    o = engine()
    o.deal_from_wall(0, build_wall([TENPAI, J1, J2, J3], draws="6p 5z 6z 7z 5p", dora="1z", ura="1s"))
    e = o.export()[0]
    assert A_RIICHI in bits(e["mask"][0])
    e = act(o, 0, {0: A_RIICHI})
    assert e["riichi_pending"] == 2 and e["cur"] == 0
    assert bits(e["mask"][0]) == [kind("3p"), kind("4p"), kind("6p")]
    e = act(o, 0, {0: kind("6p")})
    assert e["riichi"][0] == 2 and e["ippatsu"][0] == 1 and e["score"][0] == 24000 and e["kyotaku"] == 1
    assert e["riichi_idx"][0] == 0 and e["riichi_pending"] == 0 and e["delta"][0] == -1000
    e = act(o, 0, {1: kind("5z")})
    e = act(o, 0, {2: kind("6z")})
    e = act(o, 0, {3: kind("7z")})
    assert bits(e["mask"][0]) == [kind("5p"), A_TSUMO]
    e = act(o, 0, {0: A_TSUMO})
    want = (1 << 1) | (1 << 2) | (1 << 3) | (1 << 4) | (1 << 5)        # double riichi, ippatsu, tsumo, pinfu, tanyao
    assert e["yaku"][0] == want and e["han"][0] == 8 and e["fu"][0] == 20 and e["r_ura"][0] == 2
    assert e["delta"].tolist() == [25000, -8000, -8000, -8000] and e["score"][0] == 49000


def test_riichi_discard_ronned_keeps_the_stick(engine):
    o = engine()
    o.deal_from_wall(0, build_wall(["234m 34p 456p 22s 67s 5p", TENPAI2, J2, J3], draws="8s", dora="1z"))
    # seat 0: tenpai after cutting 5p (waits 2p/5p itself would be furiten, irrelevant); seat 1 wins on it
    e = act(o, 0, {0: A_RIICHI})
    assert kind("5p") in bits(e["mask"][0])
    e = act(o, 0, {0: kind("5p")})
    assert e["phase"] == 1 and e["riichi"][0] == 0 and e["score"][0] == 25000
    e = act(o, 0, {1: A_RON})
    assert e["kyotaku"] == 0 and e["delta"].tolist() == [-2000, 2000, 0, 0] and e["riichi"][0] == 0


def test_kakan_robbed(engine):
    o = engine()
    hands = ["55p 147m 28p 369s 123z", "5p 258m 39p 147s 1247z", "234m 46p 456s 22s 678s", J3]
    o2 = engine()
    o2.deal_from_wall(0, build_wall(hands, draws="4z 9m 7z 6z 5z 5p", dora="1z"))
    act(o2, 0, {0: kind("4z")}); act(o2, 0, {1: kind("5p")}); act(o2, 0, {0: A_PON, 2: A_PASS})
    act(o2, 0, {0: kind("1m")}); act(o2, 0, {1: kind("7z")}); act(o2, 0, {2: kind("6z")})
    e = act(o2, 0, {3: kind("5z")})
    assert e["cur"] == 0 and e["drawn"] == kind("5p") and A_KAN + kind("5p") in bits(e["mask"][0])
    e = act(o2, 0, {0: A_KAN + kind("5p")})
    assert e["phase"] == 2 and e["actor_mask"] == 0b0100 and bits(e["mask"][2]) == [A_RON, A_PASS]
    assert int(e["meld"][0][0]) & 7 == 5 and e["kakan_tile"] == kind("5p") and e["n_kan"] == 0
    e = act(o2, 0, {2: A_RON})
    assert e["end_type"] == 2 and e["loser"] == 0 and e["n_kan"] == 0 and e["n_dora"] == 1
    assert e["yaku"][2] == (1 << 13) | (1 << 5) and e["han"][2] == 2 and e["fu"][2] == 40     # chankan + tanyao, closed wait
    assert e["delta"].tolist() == [-2600, 0, 2600, 0]


def test_ankan_rinshan_and_new_dora(engine):
    o = engine()
    hands = ["111m 34p 456p 22s 678s", "47m258p369s1234z9m", J2, J3]
    o.deal_from_wall(0, build_wall(hands, draws="1m", rinshan="5p", dora="1z 1s"))
    e = o.export()[0]
    assert A_KAN + kind("1m") in bits(e["mask"][0])
    e = act(o, 0, {0: A_KAN + kind("1m")})
    assert e["n_kan"] == 1 and e["n_dora"] == 2 and e["rinshan"] == 1 and e["live_left"] == 68 and e["kan_by"][0] == 1
    assert int(e["meld"][0][0]) & 7 == 4 and (e["first_turn"] == 0).all()
    assert A_TSUMO in bits(e["mask"][0])
    e = act(o, 0, {0: A_TSUMO})
    # tsumo 1 + rinshan 1 + dora 2 (second indicator 1s -> 2s pair); fu 20 + 2 + 32 (concealed terminal kan) = 54 -> 60
    # 60 fu 4 han is over the 2000 cap: mangan, the dealer takes 4000 from each
    assert e["yaku"][0] == (1 << 3) | (1 << 12) and e["han"][0] == 4 and e["fu"][0] == 60 and e["r_dora"][0] == 2
    assert e["delta"].tolist() == [12000, -4000, -4000, -4000]


def test_abortive_draws(engine):
    flags = mjo.RULES_NORED | mjo.F_ABORT
    o = engine(flags=flags, mode=mjo.MODE_HALF)
    h = lambda base: "1z " + base
    o.deal_from_wall(0, build_wall([h("47m258p369s234z1m"), h("58m369p147s567z2m"), h("69m147p258s235z3m"),
                                    h("19m19p19s4567z23s")], draws="9m 9p 9s 8m"))
    e = None
    for s in range(4):
        e = act(o, 0, {s: kind("1z")})
    assert e["end_type"] == 5 and e["honba"] == 1 and e["kyoku"] == 0 and e["kyoku_serial"] == 1 and (e["delta"] == 0).all()
    # nine different terminals and honors on the first draw
    o.deal_from_wall(0, build_wall(["19m19p19s123z 2345m", J1, J2, J3], draws="4z"))
    e = o.export()[0]
    assert A_KYUUSHU in bits(e["mask"][0])
    e = act(o, 0, {0: A_KYUUSHU})
    assert e["end_type"] == 4 and e["honba"] == 2 and e["kyoku"] == 0
    # without the flag the option does not exist
    o = engine()
    o.deal_from_wall(0, build_wall(["19m19p19s123z 2345m", J1, J2, J3], draws="4z"))
    assert A_KYUUSHU not in bits(o.export()[0]["mask"][0])


def test_four_riichi_and_four_kans(engine):
    """the two abortive draws that depend on all four seats: four riichi (ends the kyoku when the fourth declaration's
    discard has gone unclaimed, its stick paid) and four kans by more than one seat (ends it after the discard that
    follows the fourth kan)"""
    flags = mjo.RULES_NORED | mjo.F_ABORT
    o = engine(flags=flags, mode=mjo.MODE_HALF)
    hands = [TENPAI, TENPAI2, "567m 34p 789p 44s 234s", "123m 789m 123s 99s 56s"]
    o.deal_from_wall(0, build_wall(hands, draws="1z 2z 3z 4z 5z"))
    e = None
    for s, t in enumerate(("1z", "2z", "3z", "4z")):
        e = act(o, 0, {s: A_RIICHI})
        e = act(o, 0, {s: kind(t)})
        if s < 3:
            assert e["end_type"] == 0 and e["kyotaku"] == s + 1 and e["cur"] == s + 1 and e["kyoku_serial"] == 0
    # every seat has paid its stick; nobody gets them back; the dealer stays, one counter more, a new deal
    assert e["end_type"] == 6 and e["honba"] == 1 and e["kyoku"] == 0 and e["kyoku_serial"] == 1 and e["kyotaku"] == 4
    assert e["score"].tolist() == [24000] * 4 and e["delta"].tolist() == [0, 0, 0, -1000] and e["terminated"] == 0
    # three riichi and an ordinary discard by the fourth seat: the kyoku goes on
    o = engine(flags=flags, mode=mjo.MODE_HALF)
    o.deal_from_wall(0, build_wall(hands, draws="1z 2z 3z 4z 5z"))
    for s, t in enumerate(("1z", "2z", "3z")):
        act(o, 0, {s: A_RIICHI})
        act(o, 0, {s: kind(t)})
    e = act(o, 0, {3: kind("4z")})
    assert e["end_type"] == 0 and e["kyoku_serial"] == 0 and e["cur"] == 0 and e["kyotaku"] == 3

    # two concealed kans each by seats 0 and 1: the discard after the fourth kan ends the kyoku
    o = engine(flags=flags, mode=mjo.MODE_HALF)
    o.deal_from_wall(0, build_wall(["1111m 4444m 345p 78p", "3333s 6666s 77m 789p", J2, J3], draws="1z 2z",
                                   rinshan="5z 6z 7z 3z"))
    e = act(o, 0, {0: A_KAN + kind("1m")})
    e = act(o, 0, {0: A_KAN + kind("4m")})
    e = act(o, 0, {0: kind("1z")})
    assert e["end_type"] == 0 and e["n_kan"] == 2 and e["cur"] == 1
    e = act(o, 0, {1: A_KAN + kind("3s")})
    e = act(o, 0, {1: A_KAN + kind("6s")})
    assert e["n_kan"] == 4 and e["end_type"] == 0 and A_KAN + kind("5z") not in bits(e["mask"][1])
    e = act(o, 0, {1: kind("2z")})
    assert e["end_type"] == 7 and e["honba"] == 1 and e["kyoku"] == 0 and e["kyoku_serial"] == 1
    assert (e["delta"] == 0).all() and e["score"].tolist() == [25000] * 4
    # all four kans by one seat: no abortive draw
    o = engine(flags=flags, mode=mjo.MODE_HALF)
    others = ["456789p 1234567s", "456789m 123p 89s 77z", "456m 789m 456p 789p 1s"]
    o.deal_from_wall(0, build_wall(["1111m 2222m 3333m 4z"] + others, draws="4z 2z", rinshan="4z 4z 5z 6z"))
    e = act(o, 0, {0: A_KAN + kind("1m")})
    e = act(o, 0, {0: A_KAN + kind("2m")})
    e = act(o, 0, {0: A_KAN + kind("3m")})
    e = act(o, 0, {0: A_KAN + kind("4z")})
    assert e["n_kan"] == 4
    e = act(o, 0, {0: kind("5z")})
    assert e["end_type"] == 0 and e["kyoku_serial"] == 0 and e["cur"] == 1


def test_bust_ends_the_game(engine):
    o = engine(mode=mjo.MODE_HALF)
    o.deal_from_wall(0, build_wall(["5p " + J1[1:], TENPAI, J2, J3], draws="1m", dora="1z"))
    e = o.export()
    e["score"][0] = [1500, 48500, 25000, 25000]
    o.import_(e)
    act(o, 0, {0: kind("5p")})
    e = act(o, 0, {1: A_RON})
    assert e["score"].tolist() == [-500, 50500, 25000, 25000] and e["terminated"] == 1 and e["kyoku"] == 0
    assert e["final_rank"].tolist() == [3, 0, 1, 2]


def _south4(o, scores, dealer_hand, winner_hand=TENPAI):
    """South 4 (the dealer is seat 3), given points; seat 3 opens by discarding 5p, which completes seat 0's hand
    (pinfu + tanyao, 2,000 from a non-dealer... paid by the dealer here)"""
    e = o.export()
    e["kyoku"][0] = 7
    e["score"][0] = scores
    o.import_(e)
    o.deal_from_wall(0, build_wall([winner_hand, J1, J2, dealer_hand], draws="1m", dora="1z", dealer=3))


def test_end_of_game_by_points(engine):
    """MJ_F_ENDGAME: 30,000 to finish, otherwise one more round; the leading dealer who repeats may stop"""
    F = mjo.RULES_NORED | mjo.F_ENDGAME
    # nobody reaches 30,000 in South 4: the game goes on into West 1 (without the flag it ends)
    for flags, over in ((F, 0), (mjo.RULES_NORED, 1)):
        o = engine(flags=flags, mode=mjo.MODE_HALF)
        _south4(o, [26000, 25000, 25000, 24000], "5p " + J3[1:])
        act(o, 0, {3: kind("5p")})
        e = act(o, 0, {0: A_RON})
        assert e["score"].tolist() == [28000, 25000, 25000, 22000] and e["terminated"] == over
        assert e["kyoku"] == (7 if over else 8)
    # somebody reaches 30,000 in South 4: over
    o = engine(flags=F, mode=mjo.MODE_HALF)
    _south4(o, [28000, 25000, 25000, 22000], "5p " + J3[1:])
    act(o, 0, {3: kind("5p")})
    e = act(o, 0, {0: A_RON})
    assert e["score"].tolist() == [30000, 25000, 25000, 20000] and e["terminated"] == 1
    assert e["final_rank"].tolist() == [0, 1, 2, 3]
    # extra round, sudden death: West 2 (kyoku 9, dealer seat 1); seat 0 wins from seat 1 and passes 30,000
    o = engine(flags=F, mode=mjo.MODE_HALF)
    e = o.export(); e["kyoku"][0] = 9; e["score"][0] = [28500, 24500, 23500, 23500]; o.import_(e)
    o.deal_from_wall(0, build_wall([TENPAI, "5p " + J1[1:], J2, J3], draws="1m", dora="1z", dealer=1))
    act(o, 0, {1: kind("5p")})
    e = act(o, 0, {0: A_RON})
    assert e["score"][0] == 30500 and e["terminated"] == 1
    # the extra round is the last: West 4 (kyoku 11, dealer seat 3) ends the game whatever the points
    o = engine(flags=F, mode=mjo.MODE_HALF)
    e = o.export(); e["kyoku"][0] = 11; e["score"][0] = [25000, 25000, 25000, 25000]; o.import_(e)
    o.deal_from_wall(0, build_wall([TENPAI, J1, J2, "5p " + J3[1:]], draws="1m", dora="1z", dealer=3))
    act(o, 0, {3: kind("5p")})
    e = act(o, 0, {0: A_RON})
    assert e["score"][0] == 27000 and e["terminated"] == 1
    # the dealer wins South 4 and is alone in the lead with 30,000: the game ends; without the flag the dealer repeats
    for flags, over in ((F, 1), (mjo.RULES_NORED, 0)):
        o = engine(flags=flags, mode=mjo.MODE_HALF)
        e = o.export(); e["kyoku"][0] = 7; e["score"][0] = [24000, 24000, 24000, 28000]; o.import_(e)
        o.deal_from_wall(0, build_wall(["5p " + J1[1:], J2, J3, TENPAI], draws="1m 9s", dora="1z", dealer=3))
        act(o, 0, {3: kind("1m")})                               # the dealer draws 1m and lets it go
        act(o, 0, {0: kind("5p")})                               # seat 0 draws 9s and discards 5p
        e = act(o, 0, {3: A_RON})                                # dealer: pinfu + tanyao = 2,900
        assert e["score"].tolist() == [21100, 24000, 24000, 30900] and e["terminated"] == over
        assert e["kyoku"] == 7 and e["honba"] == 1
    # the dealer wins South 4 but is not in the lead: play goes on with the dealer repeating
    o = engine(flags=F, mode=mjo.MODE_HALF)
    e = o.export(); e["kyoku"][0] = 7; e["score"][0] = [14000, 35000, 24000, 27000]; o.import_(e)
    o.deal_from_wall(0, build_wall(["5p " + J1[1:], J2, J3, TENPAI], draws="1m 9s", dora="1z", dealer=3))
    act(o, 0, {3: kind("1m")})
    act(o, 0, {0: kind("5p")})
    e = act(o, 0, {3: A_RON})
    assert e["score"].tolist() == [11100, 35000, 24000, 29900] and e["terminated"] == 0 and e["kyoku"] == 7


def test_late_kan_indicator(engine):
    """MJ_F_KANDORA_LATE: the indicator of an open kan waits for the seat's discard or next kan, so a win on the
    replacement tile does not count it; a concealed kan turns its indicator at once"""
    hands = [J1, "111m 34p 456p 22s 678s", J2, J3]
    wall = build_wall(hands, draws="9s", rinshan="5p", dora="1z 1s")
    for late in (False, True):
        o = engine(flags=mjo.RULES_NORED | (mjo.F_KANDORA_LATE if late else 0))
        o.deal_from_wall(0, wall)
        e = act(o, 0, {0: kind("1m")})
        assert bits(e["mask"][1]) == [A_PON, A_MINKAN, A_PASS]
        e = act(o, 0, {1: A_MINKAN})
        assert e["n_kan"] == 1 and e["rinshan"] == 1 and e["drawn"] == kind("5p")
        assert (e["n_dora"], e["dora_pending"]) == ((1, 1) if late else (2, 0))
        e = act(o, 0, {1: A_TSUMO})
        # after the kan: 34p+5p 456p 22s 678s; 20 + 2 (tsumo) + 16 (open kan of terminals) = 38 -> 40 fu;
        # rinshan 1 han, and the pair of 2s is dora only if the second indicator (1s) counts
        assert e["yaku"][1] == 1 << 12 and e["fu"][1] == 40
        if late:
            assert e["han"][1] == 1 and e["r_dora"][1] == 0 and e["delta"].tolist() == [-700, 1500, -400, -400]
        else:
            assert e["han"][1] == 3 and e["r_dora"][1] == 2 and e["delta"].tolist() == [-2600, 5200, -1300, -1300]
    # the discard after an open kan turns the indicator before the discard is answered; so does another kan
    hands = [J1, "111m 999p 34p 22s 678s", "258m 36p 1479s 4567z", J3]
    wall = build_wall(hands, draws="9s", rinshan="9p 1s", dora="1z 2z 3z")
    for second in ("discard", "kan"):
        o = engine(flags=mjo.RULES_NORED | mjo.F_KANDORA_LATE)
        o.deal_from_wall(0, wall)
        act(o, 0, {0: kind("1m")})
        e = act(o, 0, {1: A_MINKAN})
        assert (e["n_dora"], e["dora_pending"]) == (1, 1) and A_KAN + kind("9p") in bits(e["mask"][1])
        if second == "discard":
            e = act(o, 0, {1: kind("8s")})
            assert (e["n_dora"], e["dora_pending"], e["n_kan"]) == (2, 0, 1)
        else:
            e = act(o, 0, {1: A_KAN + kind("9p")})
            assert (e["n_dora"], e["dora_pending"], e["n_kan"]) == (3, 0, 2) and e["drawn"] == kind("1s")
        check_env(e, mjo.RULES_NORED | mjo.F_KANDORA_LATE)


def _play_out(o, claims=(), discards=None, tsumo=()):
    """everybody discards the tile just drawn (after a claim: the lowest legal tile) and passes on every offer, except:
    the (seat, action) pairs in `claims` are taken the first time they are offered, a seat in `discards` discards the
    listed kinds first, one per turn, and a seat in `tsumo` wins by self-draw when it can; returns the final record"""
    claims = list(claims)
    discards = {s: list(v) for s, v in (discards or {}).items()}
    for _ in range(400):
        e = o.export(0, 1)[0]
        if e["end_type"] != 0:
            assert not claims, claims
            return e
        actors = [s for s in range(4) if int(e["actor_mask"]) >> s & 1]
        moves = {}
        for s in actors:
            legal = bits(e["mask"][s])
            if e["phase"] == 0:
                d = int(e["drawn"])
                if s in tsumo and A_TSUMO in legal:
                    moves[s] = A_TSUMO
                elif discards.get(s):
                    moves[s] = discards[s].pop(0)
                else:
                    moves[s] = d if d != 255 and d in legal else min(a for a in legal if a < 34)
            else:
                take = [c for c in claims if c[0] == s and c[1] in legal]
                if take:
                    claims.remove(take[0]); moves[s] = take[0][1]
                else:
                    moves[s] = A_PASS
        act(o, 0, moves)
    raise AssertionError("the kyoku did not end")


NAGASHI_X = "5678p 2345678s 12z"            # a fourth hand from tiles the stacked draws leave over


def _nagashi_wall(seat, hands, yao="9m 9m 9m 1p 1p 1p 9p 9p 9p 1s 1s 1s 6z 6z 6z 7z 7z 7z"):
    """live draws: `seat` draws terminals and honors only, the others simples"""
    yao = yao.split()
    simples = [t for _ in range(3) for t in "2m 3m 4m 5m 6m 7m 8m 2p 3p 4p 5p 6p 7p 8p 2s 3s 4s 5s 6s 7s 8s".split()]
    draws = [yao.pop(0) if i % 4 == seat else simples.pop(0) for i in range(70)]
    return build_wall(hands, draws=" ".join(draws), dora="5z")


def test_nagashi_mangan(engine):
    """MJ_F_NAGASHI: a river of unclaimed terminals and honors is paid as a self-drawn mangan at the exhaustive draw"""
    F = mjo.RULES_NORED | mjo.F_NAGASHI
    # the dealer: 4000 from everybody; not tenpai, so the deal passes on and the counter goes up
    o = engine(flags=F, mode=mjo.MODE_HALF)
    o.deal_from_wall(0, _nagashi_wall(0, [J1, J2, J3, NAGASHI_X]))
    e = _play_out(o)
    assert e["end_type"] == 10 and e["winners"] == 0b0001 and e["tenpai_mask"] == 0
    assert e["delta"].tolist() == [12000, -4000, -4000, -4000] and e["gain"].tolist() == [12000, 0, 0, 0]
    assert e["kyoku"] == 1 and e["honba"] == 1 and e["score"].tolist() == [37000, 21000, 21000, 21000]
    # another seat: 4000 from the dealer, 2000 from the others; without the flag an ordinary exhaustive draw
    for flags in (F, mjo.RULES_NORED):
        o = engine(flags=flags, mode=mjo.MODE_HALF)
        o.deal_from_wall(0, _nagashi_wall(1, [J1, J2, J3, NAGASHI_X]))
        e = _play_out(o)
        if flags == F:
            assert e["end_type"] == 10 and e["winners"] == 0b0010 and e["delta"].tolist() == [-4000, 8000, -2000, -2000]
        else:
            assert e["end_type"] == 3 and e["winners"] == 0 and (e["delta"] == 0).all()
    # one of the discards is claimed: no payment as mangan
    o = engine(flags=F, mode=mjo.MODE_HALF)
    o.deal_from_wall(0, _nagashi_wall(0, [J1, J2, "99m 36m 147p 258s 123z", NAGASHI_X],
                                      yao="9m 9m 1m 1p 1p 1p 9p 9p 9p 1s 1s 1s 6z 6z 6z 7z 7z 7z"))
    e = _play_out(o, claims=[(2, A_PON)])
    assert e["end_type"] == 3 and e["winners"] == 0


def test_thirteen_orphans_rob_a_concealed_kan(engine):
    """MJ_F_ANKAN_ROB: only a hand waiting as thirteen orphans may win on the tile of a concealed kan"""
    hands = ["777z 234m 567p 234s 5s", "119m 19p 19s 123456z", "258m 369p 147s 4566z", J3]
    wall = build_wall(hands, draws="7z", rinshan="8s", dora="1z 2z")
    K = A_KAN + kind("7z")
    for how in ("off", "ron", "pass"):
        o = engine(flags=mjo.RULES_NORED | (0 if how == "off" else mjo.F_ANKAN_ROB))
        o.deal_from_wall(0, wall)
        e = act(o, 0, {0: K})
        if how == "off":
            assert e["phase"] == 0 and e["n_kan"] == 1 and e["n_dora"] == 2 and e["drawn"] == kind("8s")
            continue
        assert e["phase"] == 2 and e["actor_mask"] == 0b0010 and bits(e["mask"][1]) == [A_RON, A_PASS]
        assert e["kakan_tile"] == kind("7z") | 0x80 and e["n_kan"] == 0 and int(e["meld"][0][0]) & 7 == 4
        if how == "ron":
            e = act(o, 0, {1: A_RON})
            assert e["end_type"] == 2 and e["loser"] == 0 and e["winners"] == 0b0010 and e["yakuman_units"][1] == 1
            assert e["delta"].tolist() == [-32000, 32000, 0, 0]
        else:
            e = act(o, 0, {1: A_PASS})
            assert e["phase"] == 0 and e["cur"] == 0 and e["n_kan"] == 1 and e["n_dora"] == 2 and e["rinshan"] == 1
            assert e["drawn"] == kind("8s") and e["kakan_tile"] == 255 and e["furiten_temp"][1] == 1
    # an ordinary wait on the tile (78s waiting for 6s / 9s) is no offer
    hands = ["999s 234m 567p 234p 5m", "147m 258p 36s 12345z", "234m 567m 22p 78s 666z", J3]
    o = engine(flags=mjo.RULES_NORED | mjo.F_ANKAN_ROB)
    o.deal_from_wall(0, build_wall(hands, draws="9s", rinshan="1s", dora="1z 2z"))
    assert o.export()[0]["waits"][2] == (1 << kind("6s")) | (1 << kind("9s"))
    e = act(o, 0, {0: A_KAN + kind("9s")})
    assert e["phase"] == 0 and e["n_kan"] == 1 and e["furiten_temp"][2] == 0


def test_liability_for_the_three_dragons(engine):
    """MJ_F_PAO: seat 1 claims the white and the green dragon, then the red one from seat 0, who is liable from then on"""
    hands = ["147m 258p 369s 12z 57z", "55z 66z 77z 23m 11p 5s 9s 8p", J2, "369m 147p 258s 1234z"]
    plan = dict(claims=[(1, A_PON), (1, A_PON), (1, A_PON)],
                discards={0: [kind("5z"), kind("7z")], 2: [kind("6z")], 1: [kind("5s"), kind("9s"), kind("8p")]})
    F = mjo.RULES_NORED | mjo.F_PAO
    # draws in the order they happen (claims skip seats): 0, 2, 2, 3, 0, 2, 3, 0, 1
    def run(flags, draws, extra_claims=(), tsumo=()):
        o = engine(flags=flags, mode=mjo.MODE_HALF)
        o.deal_from_wall(0, build_wall(hands, draws=draws, dora="9m"))
        p = dict(plan)
        p["claims"] = plan["claims"] + list(extra_claims)
        return _play_out(o, tsumo=tsumo, **p)
    # self-draw: the liable seat pays all of it; without the flag everybody pays a share
    e = run(F, "1z 2z 3z 4z 3z 3z 4z 2z 4m", tsumo=(1,))
    assert e["end_type"] == 1 and e["yakuman_units"][1] == 1 and e["yaku"][1] == 1 << 34
    assert e["delta"].tolist() == [-32000, 32000, 0, 0]
    e = run(mjo.RULES_NORED, "1z 2z 3z 4z 3z 3z 4z 2z 4m", tsumo=(1,))
    assert e["end_type"] == 1 and e["delta"].tolist() == [-16000, 32000, -8000, -8000]
    # ron off seat 2: the liable seat and the discarder pay half each
    e = run(F, "1z 2z 3z 4z 3z 1m 4z 2z 4m", extra_claims=[(1, A_RON)])
    assert e["end_type"] == 2 and e["loser"] == 2 and e["delta"].tolist() == [-16000, 32000, -16000, 0]
    # ron off the liable seat itself: an ordinary ron
    e = run(F, "1z 2z 3z 4z 3z 3z 4z 1m 4m", extra_claims=[(1, A_RON)])
    assert e["end_type"] == 2 and e["loser"] == 0 and e["delta"].tolist() == [-32000, 32000, 0, 0]
    # a second yakuman in the same hand (all honors) is paid by all three as usual
    hands = ["147m 258p 369s 12z 57z", "55z 66z 77z 11z 22z 5s 9s 8p", J2, "3689m 147p 2458s 34z"]
    for flags, want in ((F, [-48000, 64000, -8000, -8000]), (mjo.RULES_NORED, [-32000, 64000, -16000, -16000])):
        o = engine(flags=flags, mode=mjo.MODE_HALF)
        o.deal_from_wall(0, build_wall(hands, draws="3z 4z 3z 4z 3z 9m 9m 9m 1z", dora="2s"))
        e = _play_out(o, tsumo=(1,), **plan)
        assert e["end_type"] == 1 and e["yakuman_units"][1] == 2 and e["yaku"][1] == (1 << 34) | (1 << 37)
        assert e["delta"].tolist() == want


def test_action_history(engine):
    """the kyoku's public actions in the order they took effect (action | seat << 8), and the viewer's copy of them
    with relative seats; passes are not recorded"""
    hands = ["55p 147m 28p 369s 123z", "5p 258m 39p 147s 1247z", "234m 46p 456s 22s 678s", J3]
    o = engine()
    o.deal_from_wall(0, build_wall(hands, draws="4z 9m 7z 6z 5z 5p", dora="1z"))
    script = [({0: kind("4z")}, (0, kind("4z"))), ({1: kind("5p")}, (1, kind("5p"))), ({0: A_PON, 2: A_PASS}, (0, A_PON)),
              ({0: kind("1m")}, (0, kind("1m"))), ({1: kind("7z")}, (1, kind("7z"))), ({2: kind("6z")}, (2, kind("6z"))),
              ({3: kind("5z")}, (3, kind("5z"))), ({0: A_KAN + kind("5p")}, (0, A_KAN + kind("5p"))), ({2: A_RON}, (2, A_RON))]
    want = []
    for moves, (seat, action) in script:
        e = act(o, 0, moves)
        want.append(action | seat << 8)
        assert e["n_hist"] == len(want) and e["hist"][:len(want)].tolist() == want and (e["hist"][len(want):] == 0).all()
        t = o.observe_tokens()[0]
        for me in range(4):
            assert t["n_hist"][me] == len(want) and (t["zero_"][me] == 0).all()
            assert t["hist"][me][:len(want)].tolist() == [(w & 0xFF) | (((w >> 8) - me) & 3) << 8 for w in want]
            assert (t["hist"][me][len(want):] == 0xFFFF).all()
    assert e["end_type"] == 2 and e["terminated"] == 1
    # a new kyoku starts with an empty history; a double ron is recorded in turn order from the discarder
    o = engine(mode=mjo.MODE_HALF)
    o.deal_from_wall(0, build_wall([J1, TENPAI, J2, TENPAI2], draws="5p", dora="1z"))
    e = act(o, 0, {0: kind("5p")})
    assert e["hist"][:1].tolist() == [kind("5p")] and A_RON in bits(e["mask"][1]) and A_RON in bits(e["mask"][3])
    e = act(o, 0, {1: A_RON, 3: A_RON})
    assert e["end_type"] == 2 and e["winners"] == 0b1010 and e["kyoku_serial"] == 1 and e["n_hist"] == 0 and (e["hist"] == 0).all()
    o = engine()                                   # a single kyoku: the game ends there and the history stays
    o.deal_from_wall(0, build_wall([J1, TENPAI, J2, TENPAI2], draws="5p", dora="1z"))
    act(o, 0, {0: kind("5p")})
    e = act(o, 0, {1: A_RON, 3: A_RON})
    assert e["terminated"] == 1 and e["hist"][:3].tolist() == [kind("5p"), A_RON | 1 << 8, A_RON | 3 << 8] and e["n_hist"] == 3
