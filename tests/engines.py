"""The three engines behind one interface: the CPU oracle, the host build of the kernels' per-environment
code (test-only), and the HIP library through its Python binding."""
import numpy as np


class GpuEngine:
    """adapter: numpy in / numpy out around paper_2605_20577_amd.MahjongEnv"""

    def __init__(self, B, **kw):
        import paper_2605_20577_amd as mj
        self.env = mj.MahjongEnv(B, **kw)
        self.B = B

    def step(self, actions):
        self.env.step(np.ascontiguousarray(actions, dtype=np.int8).reshape(self.B, 4))

    def sample_random(self):
        return self.env.sample_random().cpu().numpy()

    def legal_mask(self):
        return self.env.legal_mask().cpu().numpy().view(np.uint64)

    def observe(self):
        return self.env.observe().cpu().numpy()

    def observe_tokens(self):
        import paper_2605_20577_amd as mj
        return self.env.observe_tokens().cpu().numpy().view(mj.TOKEN_DTYPE).reshape(self.B, 4)

    def reward(self):
        d, r, t = self.env.reward()
        return d.cpu().numpy(), r.cpu().numpy(), t.cpu().numpy()

    def reset_done(self):
        self.env.reset_done()

    def step_random(self, n, auto_reset=True):
        self.env.step_random(n, auto_reset)

    def export(self, lo=0, n=None):
        return self.env.export(lo, n)

    def import_(self, envs, lo=0):
        self.env.import_(envs, lo)

    def deal_from_wall(self, b, wall):
        self.env.deal_from_wall(b, wall)

    def eval_hands(self, q):
        return self.env.eval_hands(q)

    def close(self):
        self.env.close()


def make_engine(kind, B, **kw):
    if kind == "oracle":
        from oracle import mjo
        return mjo.Oracle(B, **kw)
    if kind == "hostsim":
        from tests.hostsim.sim import HostSim
        return HostSim(B, **kw)
    if kind == "gpu":
        return GpuEngine(B, **kw)
    raise ValueError(kind)


def diff_records(a, b, skip=("pad_",)):
    """field-by-field difference of two canonical record arrays (dtypes may be distinct objects)"""
    out = []
    for n in a.dtype.names:
        if n in skip:
            continue
        if not np.array_equal(a[n], b[n]):
            idx = tuple(np.argwhere(a[n] != b[n])[0].tolist())
            out.append((n, idx, a[n][idx].item(), b[n][idx].item()))
    return out


def oracle_rollout_sharded(B, seed, flags, mode, steps, shards=16, with_obs=True):
    """B oracle games stepped `steps` times with the random policy, as `shards` independent oracle instances over
    consecutive env-id ranges, one thread each (the C oracle keeps no global state and ctypes drops the GIL).
    Returns the concatenated canonical records and observations (None without with_obs)."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import mjo
    bounds = [B * i // shards for i in range(shards + 1)]

    def run(i):
        lo, hi = bounds[i], bounds[i + 1]
        o = mjo.Oracle(hi - lo, seed, flags, mode, env_id_base=lo)
        o.step_random(steps)
        out = o.export().copy(), (o.observe().copy() if with_obs else None)
        o.close()
        return out
    with ThreadPoolExecutor(shards) as ex:
        parts = list(ex.map(run, range(shards)))
    return np.concatenate([p[0] for p in parts]), (np.concatenate([p[1] for p in parts]) if with_obs else None)
