"""Pins Philox, the wall shuffle and the random-policy sampler of the oracle."""
import os

import numpy as np

from oracle import mjo

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "philox_kat.txt")


def test_philox_known_answers():
    n = 0
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = [int(x, 16) for x in line.split()]
        assert mjo.philox(w[0:4], w[4:6]).tolist() == w[6:10]
        n += 1
    assert n == 3


def _philox_py(ctr, key):
    """the round function typed out again in Python integers (cross-check of operand roles)"""
    c, k = list(ctr), list(key)
    for _ in range(10):
        p0, p1 = 0xD2511F53 * c[0], 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_shuffle_definition_and_properties():
    for seed, env, serial in [(0, 0, 0), (0, 7, 3), (123, 65535, 9)]:
        w = mjo.shuffle_wall(seed, env, serial)
        assert sorted(w.tolist()) == list(range(136))
        # the definition, step by step
        r = []
        for j in range(34):
            r += _philox_py([serial, j, 0, 0], [seed, env])
        ref = list(range(136))
        for i in range(135):
            k = i + ((r[i] * (136 - i)) >> 32)
            ref[i], ref[k] = ref[k], ref[i]
        assert w.tolist() == ref
    assert (mjo.shuffle_wall(0, 1, 0) != mjo.shuffle_wall(0, 2, 0)).any()
    assert (mjo.shuffle_wall(0, 1, 0) != mjo.shuffle_wall(0, 1, 1)).any()
    assert (mjo.shuffle_wall(0, 1, 0) == mjo.shuffle_wall(0, 1, 0)).all()


def test_shuffle_uniformity():
    n = 4000
    first = np.zeros(136)
    pos_of_0 = np.zeros(136)
    for env in range(n):
        w = mjo.shuffle_wall(5, env, 0)
        first[w[0]] += 1
        pos_of_0[int(np.flatnonzero(w == 0)[0])] += 1
    for cnt in (first, pos_of_0):
        chi2 = ((cnt - n / 136) ** 2 / (n / 136)).sum()
        assert chi2 < 200, chi2          # 135 dof: mean 135, sd 16.4


def test_env_independent_of_batch_size():
    a = mjo.Oracle(16, seed=3, flags=mjo.RULES_RED, mode=mjo.MODE_HALF)
    b = mjo.Oracle(4, seed=3, flags=mjo.RULES_RED, mode=mjo.MODE_HALF, env_id_base=8)
    for _ in range(300):
        a.step_random(1)
        b.step_random(1)
    ea, eb = a.export(8, 4), b.export()
    assert ea.tobytes() == eb.tobytes()


def test_sampler_picks_legal_and_uniform():
    o = mjo.Oracle(512, seed=11)
    m = o.legal_mask()
    a = o.sample_random()
    counts = {}
    for b in range(512):
        for s in range(4):
            bits = [i for i in range(85) if int(m[b, s, i >> 6]) >> (i & 63) & 1]
            if not bits:
                assert a[b, s] == -1
                continue
            assert a[b, s] in bits
            r0 = _philox_py([0, 0, s, 1], [11, b])[0]
            assert a[b, s] == bits[(r0 * len(bits)) >> 32]
            counts.setdefault(len(bits), []).append(bits.index(a[b, s]) / len(bits))
    pos = np.concatenate([np.array(v) for v in counts.values()])
    assert 0.4 < pos.mean() < 0.6
