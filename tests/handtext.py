"""Parser for tests/golden/hands.txt (tile text -> oracle / library query records)."""
import os

import numpy as np

YAKU_BITS = {
    "riichi": 0, "driichi": 1, "ippatsu": 2, "tsumo": 3, "pinfu": 4, "tanyao": 5, "iipeikou": 6, "haku": 7,
    "hatsu": 8, "chun": 9, "seatwind": 10, "roundwind": 11, "rinshan": 12, "chankan": 13, "haitei": 14,
    "houtei": 15, "chiitoi": 16, "sanshoku": 17, "ittsu": 18, "chanta": 19, "toitoi": 20, "sanankou": 21,
    "doukou": 22, "sankantsu": 23, "honroutou": 24, "shousangen": 25, "honitsu": 26, "junchan": 27,
    "ryanpeikou": 28, "chinitsu": 29, "kokushi": 32, "suuankou": 33, "daisangen": 34, "shousuushii": 35,
    "daisuushii": 36, "tsuuiisou": 37, "chinroutou": 38, "ryuuiisou": 39, "chuuren": 40, "suukantsu": 41,
    "tenhou": 42, "chiihou": 43,
}
MELD_TYPES = {"chi": 1, "pon": 2, "minkan": 3, "ankan": 4, "kakan": 5}
FLAG_BITS = {"tsumo": 1, "ippatsu": 2, "rinshan": 4, "chankan": 8, "haitei": 16, "houtei": 32, "first": 64}
WINDS = {"E": 0, "S": 1, "W": 2, "N": 3}


def tiles(text):
    """'123m45z' -> list of kinds"""
    out, digits = [], []
    for ch in text:
        if ch.isdigit():
            digits.append(int(ch))
        else:
            base = {"m": 0, "p": 9, "s": 18, "z": 27}[ch]
            out += [base + d - 1 for d in digits]
            digits = []
    assert not digits
    return out


def parse_line(line, query_dtype):
    f = [x.strip() for x in line.split("|")]
    name, hand, melds, win, opts, expect = f
    q = np.zeros((), dtype=query_dtype)
    for k in tiles(hand):
        q["hand"][k] += 1
    n = 0
    if melds != "-":
        for m in melds.split(","):
            t, tl = m.split(":")
            ks = tiles(tl)
            q["meld"][n] = MELD_TYPES[t] | min(ks) << 3 | 1 << 9
            n += 1
    q["n_meld"] = n
    q["win_kind"] = tiles(win)[0]
    q["seat_wind"], q["round_wind"], q["kuitan"] = 1, 0, 1
    flags = 0
    if opts != "-":
        for o in opts.split(","):
            if o in FLAG_BITS:
                flags |= FLAG_BITS[o]
            elif o == "riichi":
                q["riichi"] = 1
            elif o == "driichi":
                q["riichi"] = 2
            elif o == "nokuitan":
                q["kuitan"] = 0
            elif o.startswith("seat="):
                q["seat_wind"] = WINDS[o[5:]]
            elif o.startswith("round="):
                q["round_wind"] = WINDS[o[6:]]
            elif o.startswith("dora="):
                ks = tiles(o[5:])
                q["n_ind"] = len(ks)
                q["ind"][:len(ks)] = ks
            elif o.startswith("ura="):
                ks = tiles(o[4:])
                q["ura"][:len(ks)] = ks
            elif o.startswith("aka="):
                q["n_aka"] = int(o[4:])
            else:
                raise ValueError(o)
    q["flags"] = flags
    e = expect.split()
    if e[0] == "noshape":
        exp = dict(shape_ok=0, yaku_ok=0)
    elif e[0] == "noyaku":
        exp = dict(shape_ok=1, yaku_ok=0)
    else:
        if e[0].startswith("ym="):
            units = int(e[0][3:])
            exp = dict(shape_ok=1, yaku_ok=1, yakuman_units=units, han=13 * units, fu=0, points=int(e[1]))
            names = e[2]
        else:
            exp = dict(shape_ok=1, yaku_ok=1, yakuman_units=0, han=int(e[0]), fu=int(e[1]), points=int(e[2]))
            names = e[3]
        y = 0
        for nm in names.split(","):
            y |= 1 << YAKU_BITS[nm]
        exp["yaku"] = y
    return name, q, exp


def load(query_dtype):
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "hands.txt")
    out = []
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            out.append(parse_line(line, query_dtype))
    return out
