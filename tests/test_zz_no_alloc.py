"""mj_eval_hands_static, the entry point for callers that can not allocate (no handle, no workspace: the tables sit
in a device array of the library image), against mj_eval_hands and the oracle: two calls in a row, the second with
a smaller input.  Collected last on purpose (the file name sorts after the other test files)."""
import numpy as np
import pytest

from oracle import mjo
from workloads import hands


@pytest.mark.gpu
def test_eval_hands_static_matches_eval_hands():
    import torch
    import paper_2605_20577_amd as mj
    q1 = hands.generate(5000, mj.QUERY_DTYPE, seed=11)
    q2 = hands.generate(777, mj.QUERY_DTYPE, seed=12)

    def run_static(q, dr):
        dq = torch.from_numpy(q.view(np.uint8).reshape(-1).copy()).to("cuda:0")
        mj.mj_eval_hands_static(q.size, dq, dr)
        torch.cuda.synchronize()
        return dr[:q.size * mj.RESULT_DTYPE.itemsize].cpu().numpy().view(mj.RESULT_DTYPE).copy()

    # the result buffer is reused and pre-filled, so that a stale record of the larger first call would show
    dr = torch.full((q1.size * mj.RESULT_DTYPE.itemsize,), 0xEE, dtype=torch.uint8, device="cuda:0")
    # in a fresh process these calls come before any mj_init: the first one uploads the tables itself
    s1 = run_static(q1, dr)
    dr.fill_(0xEE)
    s2 = run_static(q2, dr)
    torch.cuda.synchronize()
    tail = dr[q2.size * mj.RESULT_DTYPE.itemsize:].cpu().numpy()
    assert (tail == 0xEE).all()                                  # the smaller call wrote its own records only
    env = mj.MahjongEnv(8, seed=0, flags=mj.RULES_RED, mode=mj.MODE_HALF)
    e1, e2 = env.eval_hands(q1), env.eval_hands(q2)
    assert s1.tobytes() == e1.tobytes() and s2.tobytes() == e2.tobytes()
    assert s1.tobytes() == mjo.eval_hands(q1).tobytes() and s2.tobytes() == mjo.eval_hands(q2).tobytes()
    # and again after an mj_init on the device, larger then smaller
    assert run_static(q1, dr).tobytes() == e1.tobytes()
    assert run_static(q2, dr).tobytes() == e2.tobytes()
    # sizes: an empty batch is fine without buffers, one beyond the stated maximum is refused
    mj.mj_eval_hands_static(0, None, None)
    with pytest.raises(mj.binding.MjError, match="maximum"):
        mj.mj_eval_hands_static((1 << 24) + 1, dr, dr)
    env.close()
