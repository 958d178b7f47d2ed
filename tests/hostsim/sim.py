"""ctypes binding of the TEST-ONLY host build of the kernels' per-environment code (see hostsim.cpp).

Used by the CPU test tier to run the code of the HIP kernels against the oracle without a GPU.
Never imported by the product package.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libhostsim.so")
_CSRC = os.path.join(_HERE, "..", "..", "paper_2605_20577_amd", "csrc")

from oracle.mjo import ENV_DTYPE, QUERY_DTYPE, RESULT_DTYPE, TOKEN_DTYPE, Rules  # record layouts are the same by contract


def build(force=False):
    srcs = [os.path.join(_HERE, "hostsim.cpp")] + [os.path.join(_CSRC, f) for f in os.listdir(_CSRC) if f.endswith(".hpp")]
    srcs.append(os.path.join(_HERE, "..", "..", "include", "mj.h"))
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < max(os.path.getmtime(s) for s in srcs):
        subprocess.check_call(["g++", "-O2", "-g", "-std=c++17", "-Wno-unknown-pragmas", "-shared", "-fPIC", "-o", _SO,
                               os.path.join(_HERE, "hostsim.cpp")])
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_SO)
        vp = C.c_void_p
        L.hs_create.restype = vp
        L.hs_create.argtypes = [C.c_int64, C.c_uint64, C.POINTER(Rules)]
        L.hs_destroy.argtypes = [vp]
        L.hs_table_stats.argtypes = [vp, vp]
        L.hs_step.argtypes = [vp, vp]
        L.hs_sample.argtypes = [vp, vp]
        L.hs_reset_done.argtypes = [vp]
        L.hs_step_random.argtypes = [vp, C.c_int, C.c_int]
        L.hs_export.argtypes = [vp, C.c_int64, C.c_int64, vp]
        L.hs_import.argtypes = [vp, C.c_int64, C.c_int64, vp]
        L.hs_observe.argtypes = [vp, vp]
        L.hs_observe_tokens.argtypes = [vp, vp]
        L.hs_shanten.argtypes = [vp, vp, C.c_int]
        L.hs_shanten.restype = C.c_int
        L.hs_deal_from_wall.argtypes = [vp, C.c_int64, vp]
        L.hs_eval_hands.argtypes = [vp, C.c_int64, vp, vp]
        L.hs_waits.argtypes = [vp, vp, vp, C.c_int]
        L.hs_waits.restype = C.c_uint64
        L.hs_tenpai_discards.argtypes = [vp, vp, vp, C.c_int]
        L.hs_tenpai_discards.restype = C.c_uint64
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


class HostSim:
    def __init__(self, B, seed=0, flags=12, mode=0, start_score=25000, illegal_penalty=-1.0, env_id_base=0):
        self.B = B
        self.rules = Rules(flags, env_id_base, start_score, illegal_penalty, mode)
        self._h = C.c_void_p(lib().hs_create(B, seed, C.byref(self.rules)))

    def close(self):
        if self._h:
            lib().hs_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def table_stats(self):
        out = np.zeros(3, dtype=np.int32)
        lib().hs_table_stats(self._h, _p(out))
        return out.tolist()

    def step(self, actions):
        a = np.ascontiguousarray(actions, dtype=np.int8).reshape(self.B, 4)
        lib().hs_step(self._h, _p(a))

    def sample_random(self):
        a = np.zeros((self.B, 4), dtype=np.int8)
        lib().hs_sample(self._h, _p(a))
        return a

    def reset_done(self):
        lib().hs_reset_done(self._h)

    def step_random(self, n, auto_reset=True):
        lib().hs_step_random(self._h, n, 1 if auto_reset else 0)

    def export(self, lo=0, n=None):
        n = self.B - lo if n is None else n
        out = np.zeros(n, dtype=ENV_DTYPE)
        lib().hs_export(self._h, lo, n, _p(out))
        return out

    def import_(self, envs, lo=0):
        e = np.ascontiguousarray(envs, dtype=ENV_DTYPE)
        lib().hs_import(self._h, lo, e.size, _p(e))

    def deal_from_wall(self, b, wall):
        w = np.ascontiguousarray(wall, dtype=np.uint8)
        lib().hs_deal_from_wall(self._h, b, _p(w))

    def legal_mask(self):
        return self.export()["mask"].copy()

    def observe(self):
        o = np.zeros((self.B, 4, 56, 34), dtype=np.uint8)
        lib().hs_observe(self._h, _p(o))
        return o

    def eval_hands(self, queries):
        q = np.ascontiguousarray(queries, dtype=QUERY_DTYPE)
        r = np.zeros(q.shape, dtype=RESULT_DTYPE)
        lib().hs_eval_hands(self._h, q.size, _p(q), _p(r))
        return r

    def observe_tokens(self):
        o = np.zeros((self.B, 4), dtype=TOKEN_DTYPE)
        lib().hs_observe_tokens(self._h, _p(o))
        return o

    def shanten(self, hand, n_meld=0):
        h = np.ascontiguousarray(hand, dtype=np.uint8)
        return int(lib().hs_shanten(self._h, _p(h), n_meld))

    def waits_of(self, hand, melds=()):
        h = np.ascontiguousarray(hand, dtype=np.uint8)
        m = np.zeros(4, dtype=np.uint16)
        m[:len(melds)] = melds
        return int(lib().hs_waits(self._h, _p(h), _p(m), len(melds)))

    def tenpai_discards_of(self, hand, melds=()):
        h = np.ascontiguousarray(hand, dtype=np.uint8)
        m = np.zeros(4, dtype=np.uint16)
        m[:len(melds)] = melds
        return int(lib().hs_tenpai_discards(self._h, _p(h), _p(m), len(melds)))
