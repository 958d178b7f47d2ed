"""CPU tier: the code of the HIP kernels, compiled for the host (tests/hostsim), against the oracle.

This is the same per-environment source every kernel runs (one lane per environment); running it here lets
the GPU-less tier catch logic differences before a GPU is involved.  The GPU parity proper is test_gpu_*.py.
"""
import numpy as np
import pytest

from oracle import mjo
from tests.engines import diff_records
from tests.hostsim.sim import HostSim
from workloads import hands


def test_table_counts():
    keys, recs, rows = HostSim(1).table_stats()
    assert (keys, recs) == (21743, 23533) and rows == 98        # 97 distinct rows + the empty one


def test_hand_microbatch():
    q = hands.generate(1 << 15, mjo.QUERY_DTYPE, seed=3)
    ro, rh = mjo.eval_hands(q), HostSim(1).eval_hands(q)
    assert ro.tobytes() == rh.tobytes()
    assert ro["yaku_ok"].sum() > 5000


@pytest.mark.parametrize("flags,mode,steps", [(mjo.RULES_NORED, mjo.MODE_SINGLE, 160), (mjo.RULES_RED, mjo.MODE_HALF, 1200),
                                              (mjo.RULES_NORED | mjo.F_ABORT, mjo.MODE_EAST, 500)])
def test_rollout_trace(flags, mode, steps):
    B = 48
    o, s = mjo.Oracle(B, 7, flags, mode), HostSim(B, 7, flags, mode)
    for t in range(steps):
        d = diff_records(o.export(), s.export())
        assert not d, (t, d[:4])
        a, a2 = o.sample_random(), s.sample_random()
        assert np.array_equal(a, a2), t
        o.step(a); s.step(a)
        if t % 3 == 0:
            o.reset_done(); s.reset_done()
    assert np.array_equal(o.observe(), s.observe())


def test_fused_rollout_and_waits():
    o, s = mjo.Oracle(32, 1, mjo.RULES_RED, mjo.MODE_HALF), HostSim(32, 1, mjo.RULES_RED, mjo.MODE_HALF)
    o.step_random(700); s.step_random(700)
    eo, es = o.export(), s.export()
    assert not diff_records(eo, es)
    for b in range(32):
        for seat in range(4):
            n = int(eo["n_meld"][b, seat])
            if int(eo["hand"][b, seat].sum()) == 13 - 3 * n:
                assert s.waits_of(eo["hand"][b, seat], eo["meld"][b, seat][:n].tolist()) == int(eo["waits"][b, seat])
