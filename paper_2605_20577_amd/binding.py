"""ctypes binding of libmj.so.  Argument marshalling only."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libmj.so")

F_RED, F_ABORT, F_KUITAN, F_MULTIRON, F_ENDGAME, F_KANDORA_LATE, F_NAGASHI, F_ANKAN_ROB, F_PAO = 1, 2, 4, 8, 16, 32, 64, 128, 256
RULES_NORED = F_KUITAN | F_MULTIRON
RULES_RED = F_RED | F_ABORT | F_KUITAN | F_MULTIRON
MODE_SINGLE, MODE_EAST, MODE_HALF = 0, 1, 2
NUM_ACTIONS = 85
ROLLOUT_CHUNK = 4096          # MJ_ROLLOUT_CHUNK of include/mj.h: steps per launch of the fused path

# numpy views of the records of include/mj.h
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
TOKEN_DTYPE = np.dtype([        # MjTokenObs
    ("hand", "u1", (14,)), ("n_hand", "u1"), ("shanten", "i1"), ("drawn", "u1"), ("phase", "u1"), ("cur", "u1"),
    ("last_discarder", "u1"), ("last_discard", "u1"), ("kyoku", "u1"), ("honba", "u1"), ("kyotaku", "u1"),
    ("dealer", "u1"), ("live_left", "u1"), ("n_dora", "u1"), ("dora", "u1", (5,)), ("n_meld", "u1", (4,)),
    ("n_river", "u1", (4,)), ("riichi", "u1", (4,)), ("riichi_idx", "u1", (4,)), ("score", "<i4", (4,)),
    ("meld", "<u2", (4, 4)), ("river", "u1", (4, 32)),
    ("n_hist", "u1"), ("zero_", "u1", (15,)), ("hist", "<u2", (128,)),
])
assert ENV_DTYPE.itemsize == 1000 and QUERY_DTYPE.itemsize == 64 and RESULT_DTYPE.itemsize == 24
assert TOKEN_DTYPE.itemsize == 496


class MjRules(C.Structure):
    _fields_ = [("flags", C.c_uint32), ("env_id_base", C.c_uint32), ("start_score", C.c_int32),
                ("illegal_penalty", C.c_float), ("mode", C.c_uint8), ("pad", C.c_uint8 * 3)]


EXPORTS = {
    # name: (restype, argtypes)
    "mj_strerror": (C.c_char_p, [C.c_int]),
    "mj_state_bytes": (C.c_size_t, [C.c_int64, C.POINTER(MjRules)]),
    "mj_scratch_bytes": (C.c_size_t, [C.c_int64, C.POINTER(MjRules)]),
    "mj_init": (C.c_int, [C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p, C.c_int64, C.c_uint64, C.POINTER(MjRules),
                          C.c_void_p]),
    "mj_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "mj_step_full": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "mj_legal_mask": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "mj_observe": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "mj_observe_tokens": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "mj_reward": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "mj_standings": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "mj_reset_done": (C.c_int, [C.c_void_p, C.c_void_p]),
    "mj_sample_random": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "mj_step_random": (C.c_int, [C.c_void_p, C.c_int32, C.c_int, C.c_int, C.c_void_p, C.c_void_p]),
    "mj_export": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "mj_import": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "mj_eval_hands": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]),
    "mj_eval_hands_static": (C.c_int, [C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]),
    "mj_deal_from_wall": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]),
    "mj_step_count": (C.c_uint64, [C.c_void_p]),
    "mj_set_step_count": (C.c_int, [C.c_void_p, C.c_uint64]),
    "mj_last_step_kernel_ms": (C.c_float, [C.c_void_p]),
    "mj_destroy": (C.c_int, [C.c_void_p]),
}

_lib = None


def lib():
    """The loaded libmj.so.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            raise RuntimeError("libmj.so is not built: run `python -m paper_2605_20577_amd.build` (needs hipcc)")
        L = C.CDLL(_SO)
        for name, (res, args) in EXPORTS.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


class MjError(RuntimeError):
    pass


class _NoCtx:
    def __enter__(self):
        return self

    def __exit__(self, *exc):
        return False


_NOCTX = _NoCtx()


def _check(rc):
    if rc != 0:
        raise MjError("libmj: %s (%d)" % (lib().mj_strerror(rc).decode(), rc))


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p()


_torch = None


def _th():
    """torch, imported once (device memory and streams only)"""
    global _torch
    if _torch is None:
        import torch
        _torch = torch
    return _torch


def _stream():
    return C.c_void_p(_th().cuda.current_stream().cuda_stream)


# --- the C entry points under their own names (tensors in, nothing computed here) -------------------------
def mj_strerror(code):
    return lib().mj_strerror(code).decode()


def mj_state_bytes(B, rules):
    return lib().mj_state_bytes(B, C.byref(rules))


def mj_scratch_bytes(B, rules):
    return lib().mj_scratch_bytes(B, C.byref(rules))


def mj_init(state, scratch, B, seed, rules):
    h = C.c_void_p()
    _check(lib().mj_init(C.byref(h), _ptr(state), _ptr(scratch), B, seed, C.byref(rules), _stream()))
    return h


def mj_step(h, actions):
    _check(lib().mj_step(h, _ptr(actions), _stream()))


def mj_step_full(h, actions, auto_reset, mask=None, delta=None, reward=None, terminated=None):
    _check(lib().mj_step_full(h, _ptr(actions), int(bool(auto_reset)), _ptr(mask), _ptr(delta), _ptr(reward), _ptr(terminated),
                              _stream()))


def mj_legal_mask(h, mask):
    _check(lib().mj_legal_mask(h, _ptr(mask), _stream()))


def mj_observe(h, obs):
    _check(lib().mj_observe(h, _ptr(obs), _stream()))


def mj_observe_tokens(h, out):
    _check(lib().mj_observe_tokens(h, _ptr(out), _stream()))


def mj_standings(h, score, rank):
    _check(lib().mj_standings(h, _ptr(score), _ptr(rank), _stream()))


def mj_reward(h, delta, reward, terminated):
    _check(lib().mj_reward(h, _ptr(delta), _ptr(reward), _ptr(terminated), _stream()))


def mj_reset_done(h):
    _check(lib().mj_reset_done(h, _stream()))


def mj_sample_random(h, actions):
    _check(lib().mj_sample_random(h, _ptr(actions), _stream()))


def mj_step_random(h, n_steps, auto_reset, write_obs, obs):
    _check(lib().mj_step_random(h, n_steps, int(auto_reset), int(write_obs), _ptr(obs), _stream()))


def mj_export(h, env_lo, n, out):
    _check(lib().mj_export(h, env_lo, n, _ptr(out), _stream()))


def mj_import(h, env_lo, n, src):
    _check(lib().mj_import(h, env_lo, n, _ptr(src), _stream()))


def mj_eval_hands(h, n, queries, results):
    _check(lib().mj_eval_hands(h, n, _ptr(queries), _ptr(results), _stream()))


def mj_eval_hands_static(n, queries, results):
    _check(lib().mj_eval_hands_static(n, _ptr(queries), _ptr(results), _stream()))


def mj_deal_from_wall(h, b, wall):
    _check(lib().mj_deal_from_wall(h, b, _ptr(wall), _stream()))


def mj_destroy(h):
    _check(lib().mj_destroy(h))


def _npz_path(path):
    """numpy appends .npz to a name without it when it writes; save and restore agree on the same file"""
    path = os.fspath(path)
    return path if path.endswith(".npz") else path + ".npz"


class MahjongEnv:
    """B games on one GPU.  Owns the device buffers (torch tensors) that libmj works on."""

    def __init__(self, B, seed=0, flags=RULES_NORED, mode=MODE_SINGLE, start_score=25000, illegal_penalty=-1.0,
                 env_id_base=0, device="cuda:0"):
        torch = _th()
        self.torch = torch
        self.B = int(B)
        self.device = torch.device(device)
        if self.device.type != "cuda":
            raise MjError("libmj runs on a GPU: device %r" % (device,))
        if self.device.index is None:
            self.device = torch.device("cuda", torch.cuda.current_device())
        self._dev_index = self.device.index
        self.rules = MjRules(flags, env_id_base, start_score, illegal_penalty, mode)
        self._seed = int(seed)
        with torch.cuda.device(self.device):
            self.state = torch.empty(mj_state_bytes(B, self.rules), dtype=torch.uint8, device=self.device)
            self.scratch = torch.empty(mj_scratch_bytes(B, self.rules), dtype=torch.uint8, device=self.device)
            self._h = mj_init(self.state, self.scratch, self.B, seed, self.rules)

    def close(self):
        if getattr(self, "_h", None):
            self.torch.cuda.synchronize(self.device)
            mj_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _dev(self):
        """context that makes the environment's device current; free when it already is"""
        if self.torch.cuda.current_device() == self._dev_index:
            return _NOCTX
        return self.torch.cuda.device(self.device)

    def _want(self, t, dtype, numel, name):
        """a caller's tensor must be what the kernel will index: on this device, of this dtype, contiguous, large
        enough; anything else is refused here, before a launch could read or write out of bounds"""
        torch = self.torch
        if not torch.is_tensor(t):
            raise MjError("%s: expected a torch tensor" % name)
        if t.device != self.device:
            raise MjError("%s: tensor is on %s, the environment on %s" % (name, t.device, self.device))
        if t.dtype != dtype:
            raise MjError("%s: dtype %s, expected %s" % (name, t.dtype, dtype))
        if not t.is_contiguous():
            raise MjError("%s: tensor is not contiguous" % name)
        if t.numel() != numel:
            raise MjError("%s: %d elements, expected %d" % (name, t.numel(), numel))
        return t

    def _actions(self, actions):
        torch = self.torch
        if not torch.is_tensor(actions):
            a = np.ascontiguousarray(actions, dtype=np.int8)
            if a.size != self.B * 4:
                raise MjError("actions: %d elements, expected %d" % (a.size, self.B * 4))
            return torch.from_numpy(a.reshape(self.B, 4)).to(self.device)
        if actions.device != self.device or actions.dtype != torch.int8 or not actions.is_contiguous():
            actions = actions.to(self.device, dtype=torch.int8).contiguous()
        if actions.numel() != self.B * 4:
            raise MjError("actions: %d elements, expected %d" % (actions.numel(), self.B * 4))
        return actions

    def step(self, actions):
        a = self._actions(actions)
        with self._dev():
            mj_step(self._h, a)

    def step_full(self, actions, auto_reset=True, out=None):
        """one launch: the step, this step's (delta int32 [B,4], reward float32 [B,4], terminated uint8 [B]), the restart
        of finished games when auto_reset, and the legal mask (int64 [B,4,2]) of the state the next actions are for.
        Returns (mask, delta, reward, terminated); `out` may hold these four tensors to write into."""
        torch = self.torch
        a = self._actions(actions)
        if out is None:
            out = (torch.empty((self.B, 4, 2), dtype=torch.int64, device=self.device),
                   torch.empty((self.B, 4), dtype=torch.int32, device=self.device),
                   torch.empty((self.B, 4), dtype=torch.float32, device=self.device),
                   torch.empty((self.B,), dtype=torch.uint8, device=self.device))
        else:
            if len(out) != 4:
                raise MjError("step_full: out must hold (mask, delta, reward, terminated)")
            self._want(out[0], torch.int64, self.B * 8, "step_full mask")
            self._want(out[1], torch.int32, self.B * 4, "step_full delta")
            self._want(out[2], torch.float32, self.B * 4, "step_full reward")
            self._want(out[3], torch.uint8, self.B, "step_full terminated")
        with self._dev():
            mj_step_full(self._h, a, auto_reset, *out)
        return out

    def legal_mask(self, out=None):
        """int64 tensor [B, 4, 2] holding the two 64-bit mask words per seat"""
        torch = self.torch
        m = (self._want(out, torch.int64, self.B * 8, "legal_mask out") if out is not None
             else torch.empty((self.B, 4, 2), dtype=torch.int64, device=self.device))
        with self._dev():
            mj_legal_mask(self._h, m)
        return m

    def observe(self, out=None):
        torch = self.torch
        o = (self._want(out, torch.uint8, self.B * 4 * 56 * 34, "observe out") if out is not None
             else torch.empty((self.B, 4, 56, 34), dtype=torch.uint8, device=self.device))
        with self._dev():
            mj_observe(self._h, o)
        return o

    def observe_tokens(self, out=None):
        """token observation: uint8 tensor [B, 4, 496], one MjTokenObs per (game, viewer); view it on the host as
        TOKEN_DTYPE, or slice the byte fields on the device"""
        torch = self.torch
        o = (self._want(out, torch.uint8, self.B * 4 * TOKEN_DTYPE.itemsize, "observe_tokens out") if out is not None
             else torch.empty((self.B, 4, TOKEN_DTYPE.itemsize), dtype=torch.uint8, device=self.device))
        with self._dev():
            mj_observe_tokens(self._h, o)
        return o

    def reward(self):
        torch = self.torch
        d = torch.empty((self.B, 4), dtype=torch.int32, device=self.device)
        r = torch.empty((self.B, 4), dtype=torch.float32, device=self.device)
        t = torch.empty((self.B,), dtype=torch.uint8, device=self.device)
        with self._dev():
            mj_reward(self._h, d, r, t)
        return d, r, t

    def standings(self):
        """(points int32 [B,4], final rank uint8 [B,4]: 0 = first, meaningful for terminated games)"""
        torch = self.torch
        sc = torch.empty((self.B, 4), dtype=torch.int32, device=self.device)
        rk = torch.empty((self.B, 4), dtype=torch.uint8, device=self.device)
        with self._dev():
            mj_standings(self._h, sc, rk)
        return sc, rk

    def reset_done(self):
        with self._dev():
            mj_reset_done(self._h)

    def sample_random(self, out=None):
        torch = self.torch
        a = (self._want(out, torch.int8, self.B * 4, "sample_random out") if out is not None
             else torch.empty((self.B, 4), dtype=torch.int8, device=self.device))
        with self._dev():
            mj_sample_random(self._h, a)
        return a

    def step_random(self, n, auto_reset=True, obs=None):
        if obs is not None:
            self._want(obs, self.torch.uint8, self.B * 4 * 56 * 34, "step_random obs")
        with self._dev():
            mj_step_random(self._h, n, auto_reset, obs is not None, obs)

    def export(self, lo=0, n=None):
        """canonical records as a numpy structured array (copies to the host)"""
        torch = self.torch
        n = self.B - lo if n is None else n
        buf = torch.empty(n * ENV_DTYPE.itemsize, dtype=torch.uint8, device=self.device)
        with self._dev():
            mj_export(self._h, lo, n, buf)
        return buf.cpu().numpy().view(ENV_DTYPE).copy()

    def import_(self, envs, lo=0):
        torch = self.torch
        e = np.ascontiguousarray(envs, dtype=ENV_DTYPE)
        buf = torch.from_numpy(e.view(np.uint8).reshape(-1).copy()).to(self.device)
        with self._dev():
            mj_import(self._h, lo, e.size, buf)
            torch.cuda.current_stream().synchronize()

    def save(self, path):
        """checkpoint: the canonical records of every game, the step counter and the construction arguments
        (numpy .npz).  restore() of it continues the same trajectory, random policy included."""
        seed = int(self._seed)
        np.savez_compressed(_npz_path(path), records=self.export(), step_count=np.uint64(self.step_count), B=np.int64(self.B),
                            seed=np.uint64(seed), flags=np.uint32(self.rules.flags), mode=np.uint8(self.rules.mode),
                            env_id_base=np.uint32(self.rules.env_id_base), start_score=np.int32(self.rules.start_score),
                            illegal_penalty=np.float32(self.rules.illegal_penalty))

    @classmethod
    def restore(cls, path, device="cuda:0"):
        z = np.load(_npz_path(path), allow_pickle=False)
        env = cls(int(z["B"]), seed=int(z["seed"]), flags=int(z["flags"]), mode=int(z["mode"]),
                  start_score=int(z["start_score"]), illegal_penalty=float(z["illegal_penalty"]),
                  env_id_base=int(z["env_id_base"]), device=device)
        env.import_(z["records"])
        _check(lib().mj_set_step_count(env._h, int(z["step_count"])))
        return env

    def deal_from_wall(self, b, wall):
        torch = self.torch
        w = np.ascontiguousarray(wall, dtype=np.uint8)
        assert w.size == 136 and sorted(w.tolist()) == list(range(136))
        dw = torch.from_numpy(w.copy()).to(self.device)
        with self._dev():
            mj_deal_from_wall(self._h, b, dw)
            torch.cuda.current_stream().synchronize()

    def eval_hands(self, queries):
        torch = self.torch
        q = np.ascontiguousarray(queries, dtype=QUERY_DTYPE).reshape(-1)
        dq = torch.from_numpy(q.view(np.uint8).reshape(-1).copy()).to(self.device)
        dr = torch.empty(q.size * RESULT_DTYPE.itemsize, dtype=torch.uint8, device=self.device)
        with self._dev():
            mj_eval_hands(self._h, q.size, dq, dr)
        return dr.cpu().numpy().view(RESULT_DTYPE).copy()

    def eval_hands_device(self, dq, dr):
        """same, on records already resident on the device: uint8 tensors holding n MjHandQuery / n MjHandResult"""
        torch = self.torch
        if not torch.is_tensor(dq) or dq.numel() % QUERY_DTYPE.itemsize:
            raise MjError("eval_hands_device: the query tensor must hold whole 64-byte records")
        n = dq.numel() // QUERY_DTYPE.itemsize
        self._want(dq, torch.uint8, n * QUERY_DTYPE.itemsize, "eval_hands_device queries")
        self._want(dr, torch.uint8, n * RESULT_DTYPE.itemsize, "eval_hands_device results")
        with self._dev():
            mj_eval_hands(self._h, n, dq, dr)

    @property
    def step_count(self):
        return int(lib().mj_step_count(self._h))

    def last_step_kernel_ms(self):
        return float(lib().mj_last_step_kernel_ms(self._h))
