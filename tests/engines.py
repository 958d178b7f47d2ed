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
