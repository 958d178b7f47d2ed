#!/usr/bin/env python3
"""Benchmark of the batched Riichi Mahjong environment step on one MI355X.

Workload: B = 65,536 four-player games, no-red rules, full hanchan, uniform-random
legal policy (Philox keyed by seed, env, step, seat), auto-reset; W warm-up steps, then exactly K timed steps.
One "step" = one batched step of all B games = B env steps.  State lives in HBM before the timed region.

Prints ONE JSON line.  `value` = env steps / s of the fused sample+step+reset path (mj_step_random).
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


def timed_rollout(env, torch, warmup, steps, obs=None):
    env.step_random(warmup, True, obs)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    env.step_random(steps, True, obs)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dt, env.last_step_kernel_ms()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2048)
    ap.add_argument("--warmup", type=int, default=512)
    ap.add_argument("--batch", type=int, default=65536)
    ap.add_argument("--no-extras", action="store_true", help="skip the red-rule and observation side measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--only-obs", action="store_true",
                    help="only the configs[4] side run (B = 2^20, red rules, observation written every step), 30 steps")
    ap.add_argument("--only-tokens", action="store_true",
                    help="only the token observation of B = 2^20 games (red rules, after 60 steps), 30 launches")
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
        dt, _ = timed_rollout(env, torch, 10, 30, obs)
        print(json.dumps({"obs_B": Bo, "obs_env_steps_per_s": Bo * 30 / dt}))
        return
    env = mj.MahjongEnv(B, seed=0, flags=mj.RULES_NORED, mode=mj.MODE_HALF)
    dt, step_ms = timed_rollout(env, torch, W, K)
    value = B * K / dt
    chunk = min(K, mj.ROLLOUT_CHUNK)
    launch_ms = step_ms * chunk
    achieved = ALGO_BYTES_PER_ENV_STEP * B * chunk / (launch_ms * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "k_rollout_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("bytes_per_launch")
    out = {
        "metric": "env steps/sec on 1 MI355X (random legal policy, no-red & red); % HBM peak",
        "value": value, "unit": "env steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": dt / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": "configs[2]: B=%d games, no-red rules, full hanchan, random legal policy, auto-reset" % B,
                   "batch": B, "rules": "no-red", "mode": "half", "path": "mj_step_random (fused sample+step+reset)",
                   "steps_per_launch": chunk},
        "roofline": {"bound": "hbm", "kernel": "k_rollout", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "launch_ms": launch_ms, "algorithmic_bytes_per_env_step": ALGO_BYTES_PER_ENV_STEP},
    }
    env.close()

    if not args.no_extras:
        extras = {}
        env = mj.MahjongEnv(B, seed=0, flags=mj.RULES_RED, mode=mj.MODE_HALF)
        dt, _ = timed_rollout(env, torch, W, K)
        extras["red_rules_env_steps_per_s"] = B * K / dt
        env.close()
        # unfused API loop: sample -> step -> reset_done, three launches per step
        env = mj.MahjongEnv(B, seed=0, flags=mj.RULES_NORED, mode=mj.MODE_HALF)
        a = env.sample_random()
        n = min(K, 500)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            env.sample_random(a); env.step(a); env.reset_done()
        torch.cuda.synchronize()
        extras["unfused_api_env_steps_per_s"] = B * n / (time.perf_counter() - t0)
        # the agent loop through mj_step_full: sample -> step with rewards, restart and next mask, two launches per step
        sf = env.step_full(a, True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            env.sample_random(a); env.step_full(a, True, sf)
        torch.cuda.synchronize()
        extras["step_full_api_env_steps_per_s"] = B * n / (time.perf_counter() - t0)
        env.close()
        # configs[4]: B = 1,048,576, red rules, observation tensor written every step
        try:
            Bo = 1 << 20
            env = mj.MahjongEnv(Bo, seed=0, flags=mj.RULES_RED, mode=mj.MODE_HALF)
            obs = torch.empty((Bo, 4, 56, 34), dtype=torch.uint8, device="cuda:0")
            n = 100
            dt, _ = timed_rollout(env, torch, 20, n, obs)
            extras["obs_B"] = Bo
            extras["obs_env_steps_per_s"] = Bo * n / dt
            extras["obs_state_plus_observation_GBps"] = (OBS_BYTES_PER_ENV + ALGO_BYTES_PER_ENV_STEP) * Bo * n / dt / 1e9
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                env.observe(obs)
            torch.cuda.synchronize()
            extras["observe_kernel_GBps"] = OBS_BYTES_PER_ENV * Bo * 20 / (time.perf_counter() - t0) / 1e9
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
            dq = torch.from_numpy(q.view(np.uint8).reshape(q.size, -1)).to("cuda:0")
            dr = torch.empty((q.size, mj.RESULT_DTYPE.itemsize), dtype=torch.uint8, device="cuda:0")
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
