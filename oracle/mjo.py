"""ctypes binding of the CPU oracle (libmjo.so, built from mjo.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
cpu_baseline leg of bench.py.  The product package never imports this module.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libmjo.so")

F_RED, F_ABORT, F_KUITAN, F_MULTIRON, F_ENDGAME, F_KANDORA_LATE, F_NAGASHI, F_ANKAN_ROB, F_PAO = 1, 2, 4, 8, 16, 32, 64, 128, 256
RULES_NORED = F_KUITAN | F_MULTIRON
RULES_RED = F_RED | F_ABORT | F_KUITAN | F_MULTIRON
MODE_SINGLE, MODE_EAST, MODE_HALF = 0, 1, 2
NUM_ACTIONS = 85

ENV_DTYPE = np.dtype([
    ("discarded_kinds", "<u8", (4,)), ("waits", "<u8", (4,)), ("mask", "<u8", (4, 2)), ("yaku", "<u8", (4,)),
    ("score", "<i4", (4,)), ("delta", "<i4", (4,)), ("gain", "<i4", (4,)),
    ("episode", "<u4"), ("kyoku_serial", "<u4"),
    ("meld", "<u2", (4, 4)), ("hist", "<u2", (128,)),
    ("wall", "u1", (136,)), ("hand", "u1", (4, 34)), ("river", "u1", (4, 32)),
    ("hand_red", "u1", (4,)), ("n_meld", "u1", (4,)), ("n_river", "u1", (4,)), ("riichi_idx", "u1", (4,)),
    ("riichi", "u1", (4,)), ("ippatsu", "u1", (4,)), ("first_turn", "u1", (4,)), ("furiten_temp", "u1", (4,)),
    ("furiten_riichi", "u1", (4,)), ("kan_by", "u1", (4,)), ("final_rank", "u1", (4,)),
    ("han", "u1", (4,)), ("fu", "u1", (4,)), ("yakuman_units", "u1", (4,)),
    ("r_dora", "u1", (4,)), ("r_ura", "u1", (4,)), ("r_aka", "u1", (4,)),
    ("kyoku", "u1"), ("honba", "u1"), ("kyotaku", "u1"), ("terminated", "u1"),
    ("draw_ptr", "u1"), ("n_kan", "u1"), ("live_left", "u1"), ("n_dora", "u1"),
    ("drawn", "u1"), ("phase", "u1"), ("cur", "u1"), ("actor_mask", "u1"), ("riichi_pending", "u1"),
    ("rinshan", "u1"), ("last_discard", "u1"), ("last_discarder", "u1"), ("kakan_tile", "u1"),
    ("kuikae", "u1", (2,)), ("first_wind", "u1"), ("same_wind_cnt", "u1"), ("illegal_seat", "u1"),
    ("end_type", "u1"), ("winners", "u1"), ("loser", "u1"), ("tenpai_mask", "u1"),
    ("dora_pending", "u1"), ("n_hist", "u1"),
])

QUERY_DTYPE = np.dtype([
    ("meld", "<u2", (4,)), ("hand", "u1", (34,)), ("n_meld", "u1"), ("win_kind", "u1"), ("flags", "u1"),
    ("riichi", "u1"), ("seat_wind", "u1"), ("round_wind", "u1"), ("n_ind", "u1"),
    ("ind", "u1", (5,)), ("ura", "u1", (5,)), ("n_aka", "u1"), ("kuitan", "u1"), ("pad_", "u1", (3,)),
])
RESULT_DTYPE = np.dtype([
    ("yaku", "<u8"), ("points", "<i4"), ("han", "u1"), ("fu", "u1"), ("yakuman_units", "u1"),
    ("shape_ok", "u1"), ("yaku_ok", "u1"), ("n_dora", "u1"), ("n_ura", "u1"), ("n_aka", "u1"),
    ("pad_", "u1", (4,)),
])
TOKEN_DTYPE = np.dtype([
    ("hand", "u1", (14,)), ("n_hand", "u1"), ("shanten", "i1"), ("drawn", "u1"), ("phase", "u1"), ("cur", "u1"),
    ("last_discarder", "u1"), ("last_discard", "u1"), ("kyoku", "u1"), ("honba", "u1"), ("kyotaku", "u1"),
    ("dealer", "u1"), ("live_left", "u1"), ("n_dora", "u1"), ("dora", "u1", (5,)), ("n_meld", "u1", (4,)),
    ("n_river", "u1", (4,)), ("riichi", "u1", (4,)), ("riichi_idx", "u1", (4,)), ("score", "<i4", (4,)),
    ("meld", "<u2", (4, 4)), ("river", "u1", (4, 32)),
    ("n_hist", "u1"), ("zero_", "u1", (15,)), ("hist", "<u2", (128,)),
])
assert TOKEN_DTYPE.itemsize == 496


class Rules(C.Structure):
    _fields_ = [("flags", C.c_uint32), ("env_id_base", C.c_uint32), ("start_score", C.c_int32),
                ("illegal_penalty", C.c_float), ("mode", C.c_uint8), ("pad", C.c_uint8 * 3)]


def build(force=False):
    """Compile mjo.c with gcc (plain C11, -O2)."""
    src = os.path.join(_HERE, "mjo.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < max(
            os.path.getmtime(src), os.path.getmtime(os.path.join(_HERE, "mjo.h"))):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-shared", "-fPIC", "-o", _SO, src])
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_SO)
        vp, i64, u64, u32, i32 = C.c_void_p, C.c_int64, C.c_uint64, C.c_uint32, C.c_int32
        L.mjo_philox4x32_10.argtypes = [vp, vp, vp]
        L.mjo_shuffle_wall.argtypes = [u32, u32, u32, vp]
        L.mjo_is_complete.argtypes = [vp, C.c_int]
        L.mjo_waits_of.argtypes = [vp, vp, C.c_int]
        L.mjo_waits_of.restype = u64
        L.mjo_shanten.argtypes = [vp, C.c_int]
        L.mjo_shanten.restype = C.c_int
        L.mjo_eval_hand.argtypes = [vp, vp]
        L.mjo_create.argtypes = [C.POINTER(vp), i64, u64, C.POINTER(Rules)]
        L.mjo_step.argtypes = [vp, vp]
        L.mjo_legal_mask.argtypes = [vp, vp]
        L.mjo_observe.argtypes = [vp, vp]
        L.mjo_observe_tokens.argtypes = [vp, vp]
        L.mjo_reward.argtypes = [vp, vp, vp, vp]
        L.mjo_reset_done.argtypes = [vp]
        L.mjo_sample_random.argtypes = [vp, vp]
        L.mjo_step_random.argtypes = [vp, i32, C.c_int]
        L.mjo_export.argtypes = [vp, i64, i64, vp]
        L.mjo_import.argtypes = [vp, i64, i64, vp]
        L.mjo_deal_from_wall.argtypes = [vp, i64, vp]
        L.mjo_step_count.argtypes = [vp]
        L.mjo_step_count.restype = u64
        L.mjo_destroy.argtypes = [vp]
        L.mjo_destroy.restype = None
        L.mjo_sizeof_env.restype = C.c_size_t
        assert L.mjo_sizeof_env() == ENV_DTYPE.itemsize, (L.mjo_sizeof_env(), ENV_DTYPE.itemsize)
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def philox(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().mjo_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def shuffle_wall(seed, env_id, serial):
    w = np.zeros(136, dtype=np.uint8)
    lib().mjo_shuffle_wall(seed, env_id, serial, _p(w))
    return w


def is_complete(hand, n_meld=0):
    h = np.ascontiguousarray(hand, dtype=np.uint8)
    return bool(lib().mjo_is_complete(_p(h), n_meld))


def waits_of(hand, melds=()):
    h = np.ascontiguousarray(hand, dtype=np.uint8)
    m = np.zeros(4, dtype=np.uint16)
    m[:len(melds)] = melds
    return int(lib().mjo_waits_of(_p(h), _p(m), len(melds)))


def shanten(hand, n_meld=0):
    h = np.ascontiguousarray(hand, dtype=np.uint8)
    return int(lib().mjo_shanten(_p(h), n_meld))


def eval_hands(queries):
    q = np.ascontiguousarray(queries, dtype=QUERY_DTYPE)
    r = np.zeros(q.shape, dtype=RESULT_DTYPE)
    L = lib()
    qa, ra = q.ctypes.data, r.ctypes.data
    for i in range(q.size):
        L.mjo_eval_hand(qa + 64 * i, ra + 24 * i)
    return r


def make_meld(mtype, kind, from_rel=0, pos=0, has_red=0, called_red=0):
    return mtype | kind << 3 | from_rel << 9 | pos << 11 | has_red << 13 | called_red << 14


class Oracle:
    """B independent games stepped on the CPU."""

    def __init__(self, B, seed=0, flags=RULES_NORED, mode=MODE_SINGLE, start_score=25000,
                 illegal_penalty=-1.0, env_id_base=0):
        self.B = B
        self.rules = Rules(flags, env_id_base, start_score, illegal_penalty, mode)
        self._h = C.c_void_p()
        rc = lib().mjo_create(C.byref(self._h), B, seed, C.byref(self.rules))
        if rc != 0:
            raise ValueError("mjo_create failed: %d" % rc)

    def close(self):
        if self._h:
            lib().mjo_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step(self, actions):
        a = np.ascontiguousarray(actions, dtype=np.int8).reshape(self.B, 4)
        lib().mjo_step(self._h, _p(a))

    def legal_mask(self):
        m = np.zeros((self.B, 4, 2), dtype=np.uint64)
        lib().mjo_legal_mask(self._h, _p(m))
        return m

    def observe(self):
        o = np.zeros((self.B, 4, 56, 34), dtype=np.uint8)
        lib().mjo_observe(self._h, _p(o))
        return o

    def observe_tokens(self):
        o = np.zeros((self.B, 4), dtype=TOKEN_DTYPE)
        lib().mjo_observe_tokens(self._h, _p(o))
        return o

    def reward(self):
        d = np.zeros((self.B, 4), dtype=np.int32)
        r = np.zeros((self.B, 4), dtype=np.float32)
        t = np.zeros(self.B, dtype=np.uint8)
        lib().mjo_reward(self._h, _p(d), _p(r), _p(t))
        return d, r, t

    def reset_done(self):
        lib().mjo_reset_done(self._h)

    def sample_random(self):
        a = np.zeros((self.B, 4), dtype=np.int8)
        lib().mjo_sample_random(self._h, _p(a))
        return a

    def step_random(self, n, auto_reset=True):
        lib().mjo_step_random(self._h, n, 1 if auto_reset else 0)

    def export(self, lo=0, n=None):
        n = self.B - lo if n is None else n
        out = np.zeros(n, dtype=ENV_DTYPE)
        rc = lib().mjo_export(self._h, lo, n, _p(out))
        assert rc == 0
        return out

    def import_(self, envs, lo=0):
        e = np.ascontiguousarray(envs, dtype=ENV_DTYPE)
        rc = lib().mjo_import(self._h, lo, e.size, _p(e))
        assert rc == 0

    def deal_from_wall(self, b, wall):
        w = np.ascontiguousarray(wall, dtype=np.uint8)
        assert w.size == 136 and sorted(w.tolist()) == list(range(136))
        rc = lib().mjo_deal_from_wall(self._h, b, _p(w))
        assert rc == 0

    @property
    def step_count(self):
        return int(lib().mjo_step_count(self._h))
