#!/usr/bin/env python3
"""Benchmark of the batched Riichi Mahjong environment step on one MI355X.

Workload: B = 65,536 four-player games, no-red rules, full hanchan, uniform-random
legal policy (Philox keyed by seed, env, step, seat), auto-reset; an untimed pre-roll of 2,048 steps that brings the
batch into its steady state, W warm-up steps, then exactly K timed steps (defaults: 500 and 10,000).
One "step" = one batched step of all B games = B env steps.  State lives in HBM before the timed region.

Prints ONE JSON line.  `value` = env steps / s of the fused sample+step+reset path (mj_step_random).  `extras` holds
the configurations of the benchmark spec run literally (configs[2], [3]: 500 + 10,000 steps from fresh games; configs[4]:
2,000 steps at B = 2^20 with the observation written every step), the step-at-a-time entry points, the observation
kernels and the hand-evaluation micro-batch.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
TOKEN_BYTES_PER_ENV = 4 * 496      # token observation written per game (4 viewers)
# Algorithmic HBM bytes of one env step of the fused path: the state fields a
# step has to read and write when nothing is cached between steps, outputs included.
ALGO_BYTES_PER_ENV_STEP = 512
OBS_BYTES_PER_ENV = 4 * 56 * 34


def cpu_baseline(flags, mode, seconds_target=12.0):
    """the oracle as it stands, single thread, on a slice of the same workload"""
    from oracle import mjo
    B = 1024
    o = mjo.Oracle(B, 0, flags, mode)
    o.step_random(20)
    t0 = time.perf_counter()
    n = 0
    while True:
        o.step_random(50)
        n += 50
        dt = time.perf_counter() - t0
        if dt > seconds_target or n >= 2000:
            break
    return {"value": B * n / dt, "unit": "env steps/s", "cores": 1, "kind": "oracle",
            "sample": "B=1024 slice of the same workload (no-red, hanchan, random policy, auto-reset), %d batched steps "
                      "after 20 warm-up steps, single thread" % n}


def cpu_all_cores(flags, mode, steps=400):
    """the same oracle, one independent instance per host thread over consecutive env-id ranges (games never interact,
    and the C oracle keeps no global state; ctypes drops the GIL during a call)"""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import mjo
    threads = max(1, min(16, len(os.sched_getaffinity(0))))
    per = 256
    shards = [mjo.Oracle(per, 0, flags, mode, env_id_base=i * per) for i in range(threads)]
    for o in shards:
        o.step_random(10)
    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda o: o.step_random(steps), shards))
    dt = time.perf_counter() - t0
    return {"value": threads * per * steps / dt, "unit": "env steps/s", "cores": threads, "kind": "oracle",
            "sample": "%d shards of 256 games, %d batched steps each, one thread per shard" % (threads, steps)}


def api_loops(mj, torch, B, preroll, n=500):
    """the step-at-a-time entry points at batch B (no-red hanchan), n steps each after the pre-roll: sample -> mj_step
    -> mj_reset_done (three launches per step), and sample -> mj_step_full (two launches per step)"""
    env = mj.MahjongEnv(B, seed=0, flags=mj.RULES_NORED, mode=mj.MODE_HALF)
    if preroll:
        env.step_random(preroll)
    a = env.sample_random()
    res = {"api_steps": n}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        env.sample_random(a); env.step(a); env.reset_done()
    torch.cuda.synchronize()
    res["unfused_api_env_steps_per_s"] = B * n / (time.perf_counter() - t0)
    sf = env.step_full(a, True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        env.sample_random(a); env.step_full(a, True, sf)
    torch.cuda.synchronize()
    res["step_full_api_env_steps_per_s"] = B * n / (time.perf_counter() - t0)
    env.close()
    return res


def timed_rollout(env, torch, warmup, steps, obs=None):
    env.step_random(warmup, True, obs)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    env.step_random(steps, True, obs)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dt, env.last_step_kernel_ms()


# Every game starts at East-1 in lock step.  Before anything is timed the batch therefore runs PREROLL untimed steps
# (several hanchan under the random policy), so that the timed window, however short, sees the real mix of the
# workload: games spread over all kyoku, deals, wins, scoring, exhaustive draws and restarts.
PREROLL = 4096
ALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9      # compute units x SIMDs x lanes per cycle x clock


def protocol_run(mj, torch, B, flags, warmup, steps, obs=False):
    """a configuration of the benchmark spec run literally: fresh games, `warmup` untimed steps, `steps` timed ones"""
    env = mj.MahjongEnv(B, seed=0, flags=flags, mode=mj.MODE_HALF)
    o = torch.empty((B, 4, 56, 34), dtype=torch.uint8, device="cuda:0") if obs else None
    dt, step_ms = timed_rollout(env, torch, warmup, steps, o)
    env.close()
    del o
    return {"env_steps_per_s": B * steps / dt, "warmup": warmup, "steps": steps, "ms_per_step": dt / steps * 1e3,
            "kernel_ms_per_step": step_ms}


def rollout_counters():
    """figures of the committed rocprofv3 counter runs of k_rollout (profiles/), None when the file is missing"""
    path = os.path.join(ROOT, "profiles", "k_rollout_counters.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        return json.load(f)


def roofline_of(B, chunk, step_ms, counters):
    """roofline view of one k_rollout launch of `chunk` steps whose steps took step_ms each (HIP events)"""
    launch_ms = step_ms * chunk
    env_steps = B * chunk
    achieved = ALGO_BYTES_PER_ENV_STEP * env_steps / (launch_ms * 1e-3) / 1e9
    r = {"bound": "hbm", "kernel": "k_rollout", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": achieved / HBM_PEAK_GBS, "traffic": None, "launch_ms": launch_ms, "env_steps_per_launch": env_steps,
         "algorithmic_bytes_per_env_step": ALGO_BYTES_PER_ENV_STEP,
         "note": "achieved = algorithmic bytes (512 B per env step: the state a step reads and writes when nothing is "
                 "cached between steps) / launch time.  The kernel keeps the hot state in LDS across the steps of a "
                 "launch, so its real HBM traffic (measured_hbm) is far lower and HBM is not what binds it: vector "
                 "instruction issue under divergence is (valu)."}
    if counters:
        per = counters["hbm_bytes_per_env_step"]
        gbps = per * env_steps / (launch_ms * 1e-3) / 1e9
        r["traffic"] = per * env_steps                    # bytes per launch, like `achieved`
        r["traffic_bytes_per_env_step"] = per
        r["traffic_source"] = counters["source"]
        r["measured_hbm"] = {"GBps": gbps, "frac": gbps / HBM_PEAK_GBS}
        lane_ops = counters["valu_lane_ops_per_env_step"] * env_steps / (launch_ms * 1e-3)
        r["valu"] = {"busy_pct": counters["valu_busy_pct"], "active_lanes_per_instr": counters["active_lanes_per_valu_instr"],
                     "active_lanes_over_64": counters["active_lanes_per_valu_instr"] / 64.0,
                     "games_per_wavefront": counters["games_per_wavefront"], "waves_per_simd": counters["waves_per_simd"],
                     "lane_ops_per_s": lane_ops, "alu_peak_lane_ops_per_s": ALU_PEAK_LANE_OPS,
                     "frac_of_alu_peak": lane_ops / ALU_PEAK_LANE_OPS, "source": counters["source"]}
    return r


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10000)
    ap.add_argument("--warmup", type=int, default=500)
    ap.add_argument("--batch", type=int, default=65536)
    ap.add_argument("--rules", choices=["nored", "red"], default="nored")
    ap.add_argument("--no-preroll", action="store_true", help="start the warm-up at East-1 of every game")
    ap.add_argument("--no-extras", action="store_true", help="skip the red-rule and observation side measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--only-obs", action="store_true",
                    help="only the configs[4] side run (B = 2^20, red rules, observation written every step), 30 steps")
    ap.add_argument("--only-tokens", action="store_true",
                    help="only the token observation of B = 2^20 games (red rules, after 60 steps), 30 launches")
    ap.add_argument("--only-api", action="store_true", help="only the step-at-a-time loops (mj_step, mj_step_full), 500 steps")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 1 GiB three times (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (environments are independent, so a batch shards by env id); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2605_20577_amd as mj
    assert torch.cuda.is_available(), "needs an MI355X"
    B, K, W = args.batch, args.steps, args.warmup
    flags = mj.RULES_NORED if args.rules == "nored" else mj.RULES_RED
    if args.calibrate_copy:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30, "launches": 3}))
        return

    if args.only_tokens:
        Bo = 1 << 20
        env = mj.MahjongEnv(Bo, seed=0, flags=mj.RULES_RED, mode=mj.MODE_HALF)
        env.step_random(60)
        tok = env.observe_tokens()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(30):
            env.observe_tokens(tok)
        torch.cuda.synchronize()
        dtk = (time.perf_counter() - t0) / 30
        print(json.dumps({"tok_B": Bo, "token_observation_envs_per_s": Bo / dtk,
                          "token_observation_kernel_GBps": TOKEN_BYTES_PER_ENV * Bo / dtk / 1e9}))
        return
    if args.only_obs:
        Bo = 1 << 20
        env = mj.MahjongEnv(Bo, seed=0, flags=mj.RULES_RED, mode=mj.MODE_HALF)
        obs = torch.empty((Bo, 4, 56, 34), dtype=torch.uint8, device="cuda:0")
        if not args.no_preroll:
            env.step_random(1024)
        dt, _ = timed_rollout(env, torch, 10, 30, obs)
        print(json.dumps({"obs_B": Bo, "obs_env_steps_per_s": Bo * 30 / dt, "ms_per_step": dt / 30 * 1e3}))
        return
    if args.only_api:
        print(json.dumps(api_loops(mj, torch, B, 0 if args.no_preroll else PREROLL)))
        return

    env = mj.MahjongEnv(B, seed=0, flags=flags, mode=mj.MODE_HALF)
    preroll = 0 if args.no_preroll else PREROLL
    restarted = None
    if preroll:
        env.step_random(preroll)
        torch.cuda.synchronize()
        ep = env.export(0, min(B, 4096))
        restarted = float((ep["episode"] >= 1).mean())
        kyoku_seen = int(np.unique(ep["kyoku"]).size)
        assert restarted > 0 and kyoku_seen >= 4, "the pre-roll did not reach the steady state"
    dt, step_ms = timed_rollout(env, torch, W, K)
    value = B * K / dt
    chunk = min(K, mj.ROLLOUT_CHUNK)
    counters = rollout_counters()
    rules_name = "no-red" if args.rules == "nored" else "red"
    out = {
        "metric": "env steps/sec on 1 MI355X (random legal policy, no-red & red); % HBM peak",
        "value": value, "unit": "env steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": dt / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": "configs[%d]: B=%d games, %s rules, full hanchan, random legal policy, auto-reset"
                               % (2 if args.rules == "nored" else 3, B, rules_name),
                   "batch": B, "rules": rules_name, "mode": "half", "path": "mj_step_random (fused sample+step+reset)",
                   "steps_per_launch": chunk, "preroll_steps": preroll,
                   "preroll": "untimed steps before the warm-up, so that the timed window samples the steady state "
                              "(games spread over all kyoku, deals, wins, draws and restarts) and not East-1 of every game",
                   "games_restarted_in_preroll": restarted},
        "roofline": roofline_of(B, chunk, step_ms, counters),
    }
    # the same kernel in its full launch length, timed with HIP events outside the timed region: the figure that the
    # rocprofv3 summary under profiles/ must agree with
    env.step_random(mj.ROLLOUT_CHUNK)
    full_ms = env.last_step_kernel_ms()
    out["roofline"]["launch_full"] = {k: v for k, v in roofline_of(B, mj.ROLLOUT_CHUNK, full_ms, counters).items()
                                      if k in ("achieved", "frac", "launch_ms", "traffic", "measured_hbm")}
    out["roofline"]["launch_full"]["us_per_step"] = full_ms * 1e3
    out["roofline"]["launch_full"]["steps"] = mj.ROLLOUT_CHUNK
    env.close()

    if not args.no_extras:
        extras = {}
        # the benchmark's configurations run literally (fresh games, warm-up, timed steps)
        extras["configs2_protocol"] = protocol_run(mj, torch, 65536, mj.RULES_NORED, 500, 10000)
        extras["configs3_protocol"] = protocol_run(mj, torch, 65536, mj.RULES_RED, 500, 10000)
        extras["red_rules_env_steps_per_s"] = extras["configs3_protocol"]["env_steps_per_s"]
        extras.update(api_loops(mj, torch, B, preroll))
        # configs[4]: B = 1,048,576, red rules, observation tensor written every step, 2,000 timed steps
        try:
            Bo = 1 << 20
            c4 = protocol_run(mj, torch, Bo, mj.RULES_RED, 20, 2000, obs=True)
            extras["configs4_protocol"] = c4
            extras["obs_B"] = Bo
            extras["obs_env_steps_per_s"] = c4["env_steps_per_s"]
            extras["obs_state_plus_observation_GBps"] = (OBS_BYTES_PER_ENV + ALGO_BYTES_PER_ENV_STEP) * c4["env_steps_per_s"] / 1e9
            env = mj.MahjongEnv(Bo, seed=0, flags=mj.RULES_RED, mode=mj.MODE_HALF)
            env.step_random(300)
            obs = torch.empty((Bo, 4, 56, 34), dtype=torch.uint8, device="cuda:0")
            env.observe(obs)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                env.observe(obs)
            torch.cuda.synchronize()
            extras["observe_kernel_GBps"] = OBS_BYTES_PER_ENV * Bo * 20 / (time.perf_counter() - t0) / 1e9
            # the same kernel where configs[4] runs it: right after a step (its input no longer in the memory-side
            # cache); HIP events on the stream of the launches
            e0 = [torch.cuda.Event(enable_timing=True) for _ in range(20)]
            e1 = [torch.cuda.Event(enable_timing=True) for _ in range(20)]
            for i in range(20):
                env.step_random(1)
                e0[i].record()
                env.observe(obs)
                e1[i].record()
            torch.cuda.synchronize()
            ms = sum(a.elapsed_time(b) for a, b in zip(e0, e1)) / 20
            extras["observe_kernel_after_step_ms"] = ms
            extras["observe_kernel_after_step_GBps"] = OBS_BYTES_PER_ENV * Bo / (ms * 1e-3) / 1e9
            # the token observation of the same batch: 4 x 496 B per game, shanten number and action history included
            tok = env.observe_tokens()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                env.observe_tokens(tok)
            torch.cuda.synchronize()
            dtk = (time.perf_counter() - t0) / 20
            extras["token_observation_envs_per_s"] = Bo / dtk
            extras["token_observation_kernel_GBps"] = TOKEN_BYTES_PER_ENV * Bo / dtk / 1e9
            del tok
            env.close()
            del obs
        except Exception as ex:                                  # reported, never hidden
            extras["obs_error"] = repr(ex)
        # configs[1]: 2^20 seeded hand evaluations (yaku / han / fu / points), records resident on the device
        try:
            from workloads import hands
            q = hands.generate(1 << 20, mj.QUERY_DTYPE, seed=0)
            env = mj.MahjongEnv(64, seed=0, flags=mj.RULES_RED, mode=mj.MODE_HALF)
            dq = torch.from_numpy(q.view(np.uint8).reshape(-1).copy()).to("cuda:0")
            dr = torch.empty(q.size * mj.RESULT_DTYPE.itemsize, dtype=torch.uint8, device="cuda:0")
            for _ in range(3):
                env.eval_hands_device(dq, dr)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                env.eval_hands_device(dq, dr)
            torch.cuda.synchronize()
            extras["hand_evaluations_per_s"] = q.size * 20 / (time.perf_counter() - t0)
            env.close()
        except Exception as ex:
            extras["hands_error"] = repr(ex)
        out["extras"] = extras

    if not args.no_cpu:
        from oracle import mjo
        out["cpu_baseline"] = cpu_baseline(mjo.RULES_NORED, mjo.MODE_HALF)
        out["cpu_baseline"]["all_cores"] = cpu_all_cores(mjo.RULES_NORED, mjo.MODE_HALF)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
