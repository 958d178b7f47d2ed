"""GPU tier: the HIP library through its C ABI against the CPU oracle, bit for bit."""
import numpy as np
import pytest

from oracle import mjo
from tests.engines import GpuEngine, diff_records
from tests import handtext
from workloads import hands

pytestmark = pytest.mark.gpu


def _trace(B, seed, flags, mode, steps, reset_every=1, check_every=1, env_id_base=0):
    o = mjo.Oracle(B, seed, flags, mode, env_id_base=env_id_base)
    g = GpuEngine(B, seed=seed, flags=flags, mode=mode, env_id_base=env_id_base)
    for t in range(steps):
        if t % check_every == 0:
            d = diff_records(o.export(), g.export())
            assert not d, (t, d[:4])
            assert np.array_equal(o.legal_mask(), g.legal_mask())
        a, a2 = o.sample_random(), g.sample_random()
        assert np.array_equal(a, a2), t
        o.step(a); g.step(a)
        if t % check_every == 0:
            for x, y in zip(o.reward(), g.reward()):
                assert np.array_equal(x, y), t
        if t % reset_every == 0:
            o.reset_done(); g.reset_done()
    d = diff_records(o.export(), g.export())
    assert not d, d[:4]
    return o, g


def test_single_kyoku_full_trace():
    """B=256, no-red, one kyoku per game, every state / mask / reward of the trace until all games are over"""
    B = 256
    o = mjo.Oracle(B, 0, mjo.RULES_NORED, mjo.MODE_SINGLE)
    g = GpuEngine(B, seed=0, flags=mjo.RULES_NORED, mode=mjo.MODE_SINGLE)
    ends = None
    for t in range(400):
        eo, eg = o.export(), g.export()
        d = diff_records(eo, eg)
        assert not d, (t, d[:4])
        assert np.array_equal(o.legal_mask(), g.legal_mask())
        if eo["terminated"].all():
            ends = np.bincount(eo["end_type"], minlength=10)
            break
        a, a2 = o.sample_random(), g.sample_random()
        assert np.array_equal(a, a2)
        o.step(a); g.step(a)
        for x, y in zip(o.reward(), g.reward()):
            assert np.array_equal(x, y)
    assert ends is not None and ends[3] > 100 and ends[1] + ends[2] > 0


def test_hanchan_red_trace_with_reset_and_observation():
    o, g = _trace(192, 5, mjo.RULES_RED, mjo.MODE_HALF, 1500, reset_every=2)
    assert np.array_equal(o.observe(), g.observe())
    assert o.export()["episode"].max() >= 1


def test_east_mode_with_abortive_draws():
    _trace(128, 9, mjo.RULES_NORED | mjo.F_ABORT, mjo.MODE_EAST, 700)


@pytest.mark.parametrize("B", [1, 63, 257, 1000])
def test_ragged_batch_sizes(B):
    o, g = _trace(B, 2, mjo.RULES_RED, mjo.MODE_HALF, 150, check_every=10)
    assert np.array_equal(o.observe(), g.observe())


def test_fused_rollout_equals_unfused_and_oracle(monkeypatch):
    monkeypatch.setenv("MJ_CHUNK", "100")             # steps per launch of the fused path (default 1024)
    B = 1536
    o = mjo.Oracle(B, 4, mjo.RULES_NORED, mjo.MODE_HALF)
    g = GpuEngine(B, seed=4, flags=mjo.RULES_NORED, mode=mjo.MODE_HALF)
    for n in (1, 37, 128, 300):                       # also crosses the per-launch chunk of the fused path
        o.step_random(n); g.step_random(n)
        d = diff_records(o.export(), g.export())
        assert not d, (n, d[:4])
    assert g.env.step_count == o.step_count == 466
    # fused path with observations
    import torch
    obs = torch.zeros((B, 4, 56, 34), dtype=torch.uint8, device="cuda:0")
    o.step_random(3); g.env.step_random(3, True, obs)
    assert not diff_records(o.export(), g.export())
    assert np.array_equal(o.observe(), obs.cpu().numpy())


def test_fused_rollout_many_games():
    """4096 games, red rules, 900 fused steps with auto-reset: every field of every game against the oracle"""
    B = 4096
    o = mjo.Oracle(B, 12, mjo.RULES_RED, mjo.MODE_HALF)
    g = GpuEngine(B, seed=12, flags=mjo.RULES_RED, mode=mjo.MODE_HALF)
    for n in (450, 450):
        o.step_random(n); g.step_random(n)
        d = diff_records(o.export(), g.export())
        assert not d, (n, d[:4])
    assert np.array_equal(o.observe(), g.observe())


def test_fused_rollout_batch_in_slices():
    """110,001 games are more than the machine holds at once (65,536) and the rest fills more than half of it, so the
    fused path sends them as two launches per chunk, each over its own range of games; every field against the
    oracle after 300 steps, 150 of them in a second call"""
    from tests.engines import oracle_rollout_sharded
    B, steps = 110001, 300
    g = GpuEngine(B, seed=8, flags=mjo.RULES_RED, mode=mjo.MODE_HALF)
    g.step_random(150); g.step_random(150)
    eo, oo = oracle_rollout_sharded(B, 8, mjo.RULES_RED, mjo.MODE_HALF, steps)
    d = diff_records(eo, g.export())
    assert not d, d[:4]
    assert np.array_equal(oo, g.observe())


def test_observation_more_groups_than_resident_blocks():
    """40,003 games are 1,251 groups of 32 for the observation writer, more than the blocks it keeps resident, so every
    block takes several groups from the work counter; a second launch checks that the counters were set back"""
    B = 40003
    o = mjo.Oracle(B, 21, mjo.RULES_RED, mjo.MODE_HALF)
    g = GpuEngine(B, seed=21, flags=mjo.RULES_RED, mode=mjo.MODE_HALF)
    o.step_random(40); g.step_random(40)
    want = o.observe()
    assert np.array_equal(want, g.observe())
    assert np.array_equal(want, g.observe())
    o.step_random(5); g.step_random(5)
    assert np.array_equal(o.observe(), g.observe())


@pytest.mark.parametrize("flags,lpw,seed", [(mjo.RULES_NORED, 32, 3), (mjo.RULES_RED, 64, 4),
                                            (mjo.RULES_RED | mjo.F_ENDGAME | mjo.F_KANDORA_LATE | mjo.F_NAGASHI | mjo.F_ANKAN_ROB | mjo.F_PAO, 32, 5)])
def test_fused_rollout_large(flags, lpw, seed, monkeypatch):
    """16,384 games x 1,600 fused steps (more than a full hanchan each, so the rare paths are walked many times: wins of every
    kind, kans, robbed kans, abortive draws, busts, game ends), every field and the observation against the
    oracle, which runs as sixteen shards on the host cores"""
    from tests.engines import oracle_rollout_sharded
    monkeypatch.setenv("MJ_LPW", str(lpw))
    B, steps = 16384, 1600
    g = GpuEngine(B, seed=seed, flags=flags, mode=mjo.MODE_HALF)
    g.step_random(steps)
    eo, oo = oracle_rollout_sharded(B, seed, flags, mjo.MODE_HALF, steps)
    d = diff_records(eo, g.export())
    assert not d, d[:4]
    assert np.array_equal(oo, g.observe())


@pytest.mark.parametrize("lpw", [16, 32, 64])
def test_every_lanes_per_wave_variant(lpw, monkeypatch):
    """the step kernels exist in three variants (16 / 32 / 64 environments per wavefront); the library picks one
    by batch size, MJ_LPW forces it"""
    monkeypatch.setenv("MJ_LPW", str(lpw))
    B = 777
    o = mjo.Oracle(B, 21, mjo.RULES_RED, mjo.MODE_HALF)
    g = GpuEngine(B, seed=21, flags=mjo.RULES_RED, mode=mjo.MODE_HALF)
    o.step_random(400); g.step_random(400)
    assert not diff_records(o.export(), g.export())
    for _ in range(40):
        a = o.sample_random()
        assert np.array_equal(a, g.sample_random())
        o.step(a); g.step(a)
        o.reset_done(); g.reset_done()
    assert not diff_records(o.export(), g.export())


def test_full_size_sampled_envs():
    """B=65,536 in the benchmark's launch shape; sampled environments recomputed one by one by the oracle"""
    B, steps = 65536, 400
    for flags in (mjo.RULES_NORED, mjo.RULES_RED):
        g = GpuEngine(B, seed=0, flags=flags, mode=mjo.MODE_HALF)
        g.step_random(steps)
        rng = np.random.default_rng(1)
        ids = sorted(set([0, 1, 63, 64, 255, 256, B - 1] + rng.integers(0, B, 25).tolist()))
        for b in ids:
            o = mjo.Oracle(1, 0, flags, mjo.MODE_HALF, env_id_base=b)
            o.step_random(steps)
            d = diff_records(o.export(), g.export(b, 1))
            assert not d, (b, d[:4])
        # properties over the whole batch
        e = g.export()
        assert (e["score"].sum(1) + 1000 * e["kyotaku"].astype(np.int64) == 100000).all()
        assert (e["terminated"] == 0).all() and (e["actor_mask"] != 0).all()
        assert (e["live_left"].astype(int) == 70 - (e["draw_ptr"].astype(int) - 52) - e["n_kan"]).all()
        g.close()


@pytest.mark.parametrize("flags", [mjo.RULES_NORED, mjo.RULES_RED])
def test_full_size_every_game(flags):
    """B = 65,536 hanchan games in the benchmark's launch shape (both rule sets of the benchmark): 1,000 fused steps,
    then 200 steps through the step-at-a-time entry points (sample, step, reset) at the same size; EVERY game's
    record against the oracle, which runs the same 1,200 steps as sixteen shards on the host cores"""
    from tests.engines import oracle_rollout_sharded
    B, fused, unfused = 65536, 1000, 200
    g = GpuEngine(B, seed=0, flags=flags, mode=mjo.MODE_HALF)
    g.step_random(fused)
    a = g.env.sample_random()
    for _ in range(unfused):
        g.env.sample_random(a); g.env.step(a); g.env.reset_done()
    eo, _ = oracle_rollout_sharded(B, 0, flags, mjo.MODE_HALF, fused + unfused, with_obs=False)
    eg = g.export()
    d = diff_records(eo, eg)
    assert not d, d[:4]
    assert eg["episode"].max() >= 1 and eg["kyoku"].max() >= 6            # restarts and late kyoku were reached
    g.close()


def test_full_size_observation_workload():
    """B = 2^20, red rules, the observation written after every step (the large configuration of the benchmark, in
    its launch shape): sampled environments recomputed one by one by the oracle -- record, plane observation, token
    observation -- and whole-batch properties of the observation tensor"""
    import torch
    B, steps = 1 << 20, 12
    g = GpuEngine(B, seed=3, flags=mjo.RULES_RED, mode=mjo.MODE_HALF)
    obs = torch.zeros((B, 4, 56, 34), dtype=torch.uint8, device="cuda:0")
    g.env.step_random(steps, True, obs)
    tok = g.env.observe_tokens()
    rng = np.random.default_rng(2)
    ids = sorted(set([0, 31, 32, 65535, 65536, B - 33, B - 1] + rng.integers(0, B, 17).tolist()))
    import paper_2605_20577_amd as mj
    for b in ids:
        o = mjo.Oracle(1, 3, mjo.RULES_RED, mjo.MODE_HALF, env_id_base=b)
        o.step_random(steps)
        d = diff_records(o.export(), g.export(b, 1))
        assert not d, (b, d[:4])
        assert np.array_equal(o.observe()[0], obs[b].cpu().numpy()), b
        assert o.observe_tokens()[0].tobytes() == tok[b].cpu().numpy().tobytes(), b
    # every byte is 0 or 1; the own-hand planes of a viewer count 13 or 14 tiles minus three per meld
    assert int(obs.max()) == 1
    hand_tiles = obs[:, :, 0:4, :].sum(dim=(2, 3), dtype=torch.int32).cpu().numpy()
    e = g.export()
    expect = 13 - 3 * e["n_meld"].astype(np.int32)
    turn = (e["phase"] == 0) & (e["drawn"] != 255)
    expect[np.arange(B)[turn], e["cur"][turn]] += 1
    after_call = (e["phase"] == 0) & (e["drawn"] == 255)            # a claim: the seat to move holds one tile more
    expect[np.arange(B)[after_call], e["cur"][after_call]] += 1
    assert np.array_equal(hand_tiles, expect)
    # the fused path over the same batch: one launch, sixteen times what the machine holds at once
    g.step_random(300)
    # ... and both observations again, now that rivers and melds have filled up
    g.env.observe(obs)
    tok = g.env.observe_tokens(tok)
    for b in ids[::3]:
        o = mjo.Oracle(1, 3, mjo.RULES_RED, mjo.MODE_HALF, env_id_base=b)
        o.step_random(steps + 300)
        d = diff_records(o.export(), g.export(b, 1))
        assert not d, (b, d[:4])
        assert np.array_equal(o.observe()[0], obs[b].cpu().numpy()), b
        assert o.observe_tokens()[0].tobytes() == tok[b].cpu().numpy().tobytes(), b
    g.close()


@pytest.mark.parametrize("mode,auto_reset", [(mjo.MODE_SINGLE, True), (mjo.MODE_HALF, True), (mjo.MODE_EAST, False)])
def test_step_full_equals_the_separate_calls(mode, auto_reset):
    """mj_step_full hands back in one launch what step + reward + reset_done + legal_mask give on the oracle"""
    B = 321
    o = mjo.Oracle(B, 6, mjo.RULES_RED, mode)
    g = GpuEngine(B, seed=6, flags=mjo.RULES_RED, mode=mode)
    ended = 0
    for t in range(260):
        a = o.sample_random()
        if t == 100:
            a[7, :] = 84                              # an illegal action somewhere: the penalty must show in the reward
        o.step(a)
        want = o.reward()
        if auto_reset:
            o.reset_done()
        mask, delta, reward, term = [x.cpu().numpy() for x in g.env.step_full(a, auto_reset)]
        assert np.array_equal(delta, want[0]) and np.array_equal(reward, want[1]) and np.array_equal(term, want[2]), t
        assert np.array_equal(mask.view(np.uint64), o.legal_mask()), t
        ended += int(want[2].sum())
    assert not diff_records(o.export(), g.export())
    assert ended > 0


def test_import_export_roundtrip():
    o = mjo.Oracle(64, 8, mjo.RULES_RED, mjo.MODE_HALF)
    o.step_random(333)
    g = GpuEngine(64, seed=8, flags=mjo.RULES_RED, mode=mjo.MODE_HALF)
    g.import_(o.export())
    assert not diff_records(o.export(), g.export())
    # continue from the imported state: the step counters differ, so drive both with the oracle's actions
    for _ in range(100):
        a = o.sample_random()
        o.step(a); g.step(a)
        o.reset_done(); g.reset_done()
    d = diff_records(o.export(), g.export())
    assert not d, d[:4]


def test_illegal_action():
    o, g = mjo.Oracle(8, 1), GpuEngine(8, seed=1)
    a = o.sample_random()
    a[3, int(o.export()["cur"][3])] = 74          # RON on the own turn
    a[5, :] = -1
    o.step(a); g.step(a)
    assert not diff_records(o.export(), g.export())
    for x, y in zip(o.reward(), g.reward()):
        assert np.array_equal(x, y)
    assert g.reward()[1][3].min() == -1.0 and g.export()["end_type"][3] == 9


def test_worked_hands_on_gpu():
    g = GpuEngine(1)
    cases = handtext.load(mjo.QUERY_DTYPE)
    r = g.eval_hands(np.array([c[1] for c in cases]))
    for (name, q, exp), got in zip(cases, r):
        for k, v in exp.items():
            assert int(got[k]) == v, (name, k, int(got[k]), v)


def test_hand_microbatch_full_size():
    """2^20 hands on the GPU; all of them against the oracle"""
    g = GpuEngine(1)
    q = hands.generate(1 << 20, mjo.QUERY_DTYPE, seed=0)
    rg = g.eval_hands(q)
    ro = mjo.eval_hands(q)
    bad = np.flatnonzero((ro.view(np.uint8).reshape(-1, 24) != rg.view(np.uint8).reshape(-1, 24)).any(1))
    assert bad.size == 0, (bad[:5], ro[bad[:2]], rg[bad[:2]])
    assert ro["yaku_ok"].sum() > 250000 and (ro["yakuman_units"] > 0).sum() > 1000
    # edge cases: empty batch, ragged tail
    assert g.eval_hands(q[:0]).size == 0
    assert g.eval_hands(q[:257]).tobytes() == ro[:257].tobytes()


def test_standings_match_the_records():
    B = 600
    o = mjo.Oracle(B, 5, mjo.RULES_RED, mjo.MODE_EAST)
    g = GpuEngine(B, seed=5, flags=mjo.RULES_RED, mode=mjo.MODE_EAST)
    o.step_random(700, auto_reset=False); g.step_random(700, auto_reset=False)
    eo = o.export()
    assert eo["terminated"].sum() > B // 2                       # most east games are over by now
    score, rank = g.env.standings()
    assert np.array_equal(score.cpu().numpy(), eo["score"])
    assert np.array_equal(rank.cpu().numpy(), eo["final_rank"])


def _oracle_play(o, policies, n_games):
    """tests' restatement of arena.play on the oracle, in numpy"""
    B = o.B
    rank_count = np.zeros((4, 4), dtype=np.int64)
    done = steps = 0
    while done < n_games:
        words = o.legal_mask().reshape(B, 4, 2)
        bits = ((words[..., None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(bool).reshape(B, 4, 128)[:, :, :85]
        actions = np.full((B, 4), -1, dtype=np.int8)
        for s, pol in enumerate(policies):
            a = pol(bits[:, s])
            acts = bits[:, s].any(axis=1)
            actions[acts, s] = a[acts]
        o.step(actions)
        steps += 1
        term = o.reward()[2]
        idx = np.flatnonzero(term)[: n_games - done]
        if idx.size:
            r = o.export()["final_rank"][idx]
            for s in range(4):
                rank_count[s] += np.bincount(r[:, s], minlength=4)
            done += idx.size
            o.reset_done()
    return rank_count, steps


def test_one_vs_three_evaluation_matches_the_oracle():
    """section 4.2's protocol (one agent against three fixed opponents, rated by average rank) with two
    deterministic policies: the harness on the HIP library and the same loop on the oracle see the same games"""
    from paper_2605_20577_amd import arena
    B, n_games = 96, 150
    g = GpuEngine(B, seed=9, flags=mjo.RULES_RED, mode=mjo.MODE_EAST)
    res = arena.one_vs_three(g.env, arena.highest_legal, arena.lowest_legal, n_games)
    o = mjo.Oracle(B, 9, mjo.RULES_RED, mjo.MODE_EAST)
    hi = lambda m: 84 - np.argmax(m[:, ::-1], axis=1)
    lo = lambda m: np.argmax(m, axis=1)
    rank_count, steps = _oracle_play(o, [hi, lo, lo, lo], n_games)
    assert res["games"] == n_games and res["steps"] == steps
    assert np.array_equal(np.array(res["rank_count"]), rank_count)
    assert abs(sum(res["mean_rank"]) - 10.0) < 1e-9               # ranks 1..4 are shared out in every game
    assert not diff_records(o.export(), g.export())


def test_checkpoint_and_resume(tmp_path):
    """records + step counter saved after 300 steps and restored into a fresh library instance continue exactly
    like the run that was never interrupted (and like the oracle)"""
    import paper_2605_20577_amd as mj
    B = 500
    g = GpuEngine(B, seed=31, flags=mjo.RULES_RED, mode=mjo.MODE_HALF)
    g.step_random(300)
    path = str(tmp_path / "ckpt.npz")
    g.env.save(path)
    g.step_random(400)
    r = mj.MahjongEnv.restore(path)
    assert r.step_count == 300
    r.step_random(400)
    assert not diff_records(g.export(), r.export())
    o = mjo.Oracle(B, 31, mjo.RULES_RED, mjo.MODE_HALF)
    o.step_random(700)
    assert not diff_records(o.export(), r.export())
    assert np.array_equal(o.observe(), r.observe().cpu().numpy())
    r.close()


@pytest.mark.parametrize("B,flags,mode", [(1, mjo.RULES_RED, mjo.MODE_HALF), (257, mjo.RULES_NORED, mjo.MODE_EAST),
                                          (3000, mjo.RULES_RED, mjo.MODE_HALF)])
def test_token_observation(B, flags, mode):
    """the token observation (hand tokens, shanten number, rivers, melds, scalars) of every viewer against the
    oracle's, along a rollout"""
    o = mjo.Oracle(B, 17, flags, mode)
    g = GpuEngine(B, seed=17, flags=flags, mode=mode)
    shanten_seen = set()
    for n in (0, 1, 40, 150, 400, 409):
        o.step_random(n); g.step_random(n)
        want = o.observe_tokens()
        got = g.env.observe_tokens().cpu().numpy().reshape(B, 4, -1).view(mjo.TOKEN_DTYPE).reshape(B, 4)
        for name in want.dtype.names:
            assert np.array_equal(want[name], got[name]), (n, name)
        shanten_seen |= set(np.unique(want["shanten"]).tolist())
    if B >= 3000:
        assert {-1, 0, 1, 2, 3, 4, 5} <= shanten_seen


def test_binding_refuses_tensors_the_kernels_could_not_index():
    """a caller's tensor of the wrong size, dtype or device is refused on the host, before any launch"""
    import torch
    import paper_2605_20577_amd as mj
    env = mj.MahjongEnv(100, seed=0)
    with pytest.raises(mj.binding.MjError):
        env.step(torch.zeros((99, 4), dtype=torch.int8, device="cuda:0"))
    with pytest.raises(mj.binding.MjError):
        env.observe(torch.empty((100, 4, 56, 33), dtype=torch.uint8, device="cuda:0"))
    with pytest.raises(mj.binding.MjError):
        env.legal_mask(torch.empty((100, 4, 2), dtype=torch.int32, device="cuda:0"))
    with pytest.raises(mj.binding.MjError):
        env.sample_random(torch.empty((100, 4), dtype=torch.int8))
    with pytest.raises(mj.binding.MjError):
        env.observe_tokens(torch.empty((100, 4, 496), dtype=torch.uint8, device="cuda:0")[:, :, ::2])
    env.step(env.sample_random())                        # and the environment still works
    env.close()


@pytest.mark.parametrize("B", [33, 3000])
def test_fused_steps_with_observation_every_step(B):
    """the fused path with write_obs: the bit strings of a step are expanded on the library's second stream while the
    next step runs; after each call (1, 2, 5, 3 and 64 steps, two calls back to back without a synchronisation in
    between) the tensor holds the observation of the last step, and the state is the oracle's"""
    import torch
    o = mjo.Oracle(B, 14, mjo.RULES_RED, mjo.MODE_HALF)
    g = GpuEngine(B, seed=14, flags=mjo.RULES_RED, mode=mjo.MODE_HALF)
    obs = torch.zeros((B, 4, 56, 34), dtype=torch.uint8, device="cuda:0")
    for n in (1, 2, 5, 3, 64):
        g.env.step_random(n, True, obs)
        o.step_random(n)
        assert np.array_equal(o.observe(), obs.cpu().numpy()), n
    g.env.step_random(7, True, obs)
    g.env.step_random(4, True, obs)
    o.step_random(11)
    assert np.array_equal(o.observe(), obs.cpu().numpy())
    assert not diff_records(o.export(), g.export())
    # the separate entry point still agrees
    assert np.array_equal(o.observe(), g.observe())
    g.close()


@pytest.mark.parametrize("mode,auto_reset", [(mjo.MODE_HALF, True), (mjo.MODE_SINGLE, False)])
def test_action_history_across_launches(mode, auto_reset):
    """The fused kernel collects a game's action history in LDS and writes it out every 32 steps, before a shuffle
    takes the column, and at the end of a launch; the one-step kernels store entry by entry.  Launches of every length
    around those intervals, mixed with step-at-a-time calls, restarts inside a launch and games that stay finished:
    the history of the record and of the token observation against the oracle after each."""
    B = 700
    o = mjo.Oracle(B, 23, mjo.RULES_RED, mode)
    g = GpuEngine(B, seed=23, flags=mjo.RULES_RED, mode=mode)
    def check(tag):
        a, b = o.export(), g.export()
        assert np.array_equal(a["n_hist"], b["n_hist"]), tag
        assert np.array_equal(a["hist"], b["hist"]), tag
        d = diff_records(a, b)
        assert not d, (tag, d[:4])
        want = o.observe_tokens()
        got = g.env.observe_tokens().cpu().numpy().reshape(B, 4, -1).view(mjo.TOKEN_DTYPE).reshape(B, 4)
        assert np.array_equal(want["n_hist"], got["n_hist"]) and np.array_equal(want["hist"], got["hist"]), tag
    for n in (1, 2, 29, 1, 31, 32, 33, 1, 63, 64, 65, 7, 130, 1, 1, 250):
        o.step_random(n, auto_reset); g.env.step_random(n, auto_reset)
        check(("fused", n))
        for _ in range(3):                                        # step-at-a-time calls in between
            a = o.sample_random()
            o.step(a); g.step(a)
            if auto_reset:
                o.reset_done(); g.reset_done()
        check(("stepwise after", n))
    assert o.export()["n_hist"].max() > 40


@pytest.mark.skipif(not __import__("os").environ.get("MJ_TEST_HUGE"),
                    reason="4.5 minutes of host time: set MJ_TEST_HUGE=1 to run it")
def test_largest_batch_every_game():
    """every one of 2^20 games (red rules, hanchan) after 600 fused steps, in launches of 512 steps as the library
    chooses for this batch size, field by field against the oracle (128 shards of 8,192 games on 16 host threads)"""
    from concurrent.futures import ThreadPoolExecutor
    B, steps, shard = 1 << 20, 600, 8192
    g = GpuEngine(B, seed=5, flags=mjo.RULES_RED, mode=mjo.MODE_HALF)
    g.step_random(steps)
    got = g.export()

    def run(i):
        lo, hi = i * shard, (i + 1) * shard
        o = mjo.Oracle(hi - lo, 5, mjo.RULES_RED, mjo.MODE_HALF, env_id_base=lo)
        o.step_random(steps)
        d = diff_records(o.export(), got[lo:hi])
        o.close()
        return i, d
    with ThreadPoolExecutor(16) as ex:
        for i, d in ex.map(run, range(B // shard)):
            assert not d, (i, d[:4])
            if i % 16 == 15:
                print("largest batch: %d of %d shards identical" % (i + 1, B // shard), flush=True)   # seen with -s
