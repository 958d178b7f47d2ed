"""Pins the oracle's hand evaluator to hand-computed values (tests/golden/hands.txt)."""
import numpy as np
import pytest

from oracle import mjo
from tests import handtext

CASES = handtext.load(mjo.QUERY_DTYPE)


@pytest.mark.parametrize("name,q,exp", CASES, ids=[c[0] for c in CASES])
def test_worked_hand(name, q, exp):
    r = mjo.eval_hands(q.reshape(1))[0]
    for k, v in exp.items():
        assert int(r[k]) == v, (name, k, int(r[k]), v, {n: int(r[n]) if r[n].shape == () else r[n] for n in r.dtype.names})
    if not exp["yaku_ok"]:
        assert r["points"] == 0 and r["han"] == 0 and r["yaku"] == 0
