#!/usr/bin/env python3
"""Throughput of the TABX batched tick (fused step + observe) on one MI355X.

A "step" is one tick of the whole hot path for every env of the workload: physics,
actions, hurtbox combat, zones, rewards, termination with auto-reset, and the per-agent
observations.  Inputs (scenario, pre-generated seeded actions) are resident in HBM before
the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published

def measured_traffic(workload: str):
    """HBM bytes per launch of the fused tick as the committed rocprofv3 summary of that workload
    states them (`profiles/tabx_tick_<workload>.md`, line `traffic_bytes_per_launch: N (commit C)`:
    FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reads for a plain copy).  They
    are measurements of the commit named there, not of this run: None if there is no summary."""
    import re
    path = os.path.join(ROOT, "profiles", f"tabx_tick_{workload}.md")
    try:
        m = re.search(r"traffic_bytes_per_launch:\s*(\d+)\s*\(commit\s+(\w+)\)", open(path).read())
    except OSError:
        return None, None
    if not m:
        return None, None
    return int(m.group(1)), {"file": os.path.relpath(path, ROOT), "commit": m.group(2)}


def algorithmic_bytes_per_env(N: int, D: int, Z: int) -> int:
    """Bytes one env-tick must move (fused step + observe): obs write, state read+write,
    specs, action, reward, action mask, terrain cell, visibility mask per unit; zone
    descriptors, tick counter / potential / done per env."""
    words = (N + 63) // 64
    per_unit = 4 * D + 2 * 37 + 46 + 1 + 4 + 1 + 1 + 8 * words
    return N * per_unit + 24 * Z + 17


def cpu_baseline(w, I, scenario: dict, sample_envs: int, ticks: int) -> dict:
    """The CPU checker as it stands, timed on a bounded sample of the workload: once on one
    thread, once with the sample's envs dealt to one thread per host core (envs share nothing;
    the checker itself stays single-threaded, each thread steps its own sub-batch through it)."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    from oracle.ref import RefEnv
    E = min(sample_envs, w.num_envs)
    N = w.num_units
    acts = [I.actions_for_step(w.seed, s, E, N) for s in range(min(ticks, 64))]

    def run(lo, hi, n_ticks):
        env = RefEnv(I.make_params(w, hi - lo), I.take_envs(scenario, slice(lo, hi)))
        env.reset()
        part = [np.ascontiguousarray(a[lo:hi]) for a in acts]
        t0 = time.perf_counter()
        for s in range(n_ticks):
            env.step(part[s % len(part)])
            env.observe()
        return time.perf_counter() - t0

    import numpy as np
    single_ticks = max(1, ticks // 4)
    dt1 = run(0, E, single_ticks)
    single = E * N * single_ticks / dt1
    # one thread per core of this job's CPU share: the GPU machines export it as OMP_NUM_THREADS (a
    # one-GPU job may use 16 of the host's cores, whatever os.cpu_count() shows); else every core
    host_cores = os.cpu_count() or 1
    share = int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or host_cores
    cores = max(1, min(share, host_cores, E))
    bounds = [E * k // cores for k in range(cores + 1)]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as pool:     # the checker's calls release the interpreter lock
        list(pool.map(lambda k: run(bounds[k], bounds[k + 1], ticks), range(cores)))
    dt = time.perf_counter() - t0
    return {"value": E * N * ticks / dt, "unit": "agent-steps/s", "cores": cores,
            "host_cores": host_cores, "kind": "oracle", "single_thread_value": single,
            "sample": f"first {E} envs of the workload: {ticks} ticks of step+observe on "
                      f"{cores} threads ({dt:.1f} s), {single_ticks} ticks on one ({dt1:.1f} s)"}


def time_workload(I, TabxEnv, torch, name: str, ticks: int, warmup: int) -> dict:
    """The fused tick of one more workload, timed with HIP events on the launch stream: `ticks`
    ticks after `warmup`, a fresh pre-generated action batch per tick."""
    w = I.WORKLOADS[name]
    E, N = w.num_envs, w.num_units
    p = I.make_params(w)
    env = TabxEnv(p, I.make_scenario(w))
    env.reset()
    n_act = max(1, min(ticks + warmup, (1 << 28) // (E * N)))
    acts = [torch.from_numpy(I.actions_for_step(w.seed, s, E, N)).to("cuda:0") for s in range(n_act)]
    stream = torch.cuda.current_stream()
    for s in range(warmup):
        env.step_observe(acts[s % n_act], stream)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for s in range(ticks):
        env.step_observe(acts[(warmup + s) % n_act], stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert torch.isfinite(env.obs).all()
    ms = ev0.elapsed_time(ev1) / ticks
    B = algorithmic_bytes_per_env(N, env.D, p["max_zones"]) * E
    gbs = B / (ms * 1e-3) / 1e9
    return {"num_envs": E, "units_per_env": N, "obs_dim": env.D, "ticks": ticks, "warmup": warmup,
            "ms_per_step": wall * 1e3 / ticks, "kernel_ms": ms,
            "agent_steps_per_s": E * N * ticks / wall,
            "algorithmic_bytes_per_launch": B, "algorithmic_GBs": gbs,
            "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed ticks (default: the workload's own step count, 1000 for the headline)")
    ap.add_argument("--warmup", type=int, default=300,
                    help="untimed ticks before the timed region (the clocks of an idle GPU take a few ms to settle)")
    ap.add_argument("--workload", default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="also time a plain device fill and copy of the obs-sized buffer "
                         "(reference points for the HBM roofline and for rocprofv3 byte counters)")
    ap.add_argument("--collisions", action="store_true",
                    help="switch the optional body-collision correction on (alpha 0.8, slop 0.01); "
                         "not part of the headline tick")
    ap.add_argument("--dynamics", action="store_true",
                    help="persistent velocities with the collision impulse (TabxParams.dynamics = 1, "
                         "move_gain 2, restitution 0.5; implies --collisions); not the headline tick")
    ap.add_argument("--separate", action="store_true",
                    help="time tabx_step + tabx_observe as two launches instead of the fused one")
    ap.add_argument("--reps", type=int, default=5,
                    help="timed regions of --steps ticks each; the first gives `value`, all of "
                         "them the median / min kernel time reported in `roofline`")
    ap.add_argument("--policy", default=None, metavar="TIER",
                    help="the adversaries are moved by the heuristic policy of this tier inside "
                         "the tick launch (tabx_scripted_step_observe: they decide in the observe "
                         "stage); with --separate as tabx_heuristic_actions + tabx_step_observe, "
                         "with --policy-scan as tabx_policy_step_observe; not the headline tick")
    ap.add_argument("--global-state", action="store_true",
                    help="also have every tick write the global state (TabxState.global_state), "
                         "as a centralised critic would want it; not the headline tick")
    ap.add_argument("--action-batches", type=int, default=None,
                    help="distinct pre-generated action batches (default: one per tick, at most "
                         "1 GiB of them); fewer are cycled")
    ap.add_argument("--streams", type=int, default=2,
                    help="also time the tick with the batch split into this many parts, each "
                         "launched on a stream of its own (reported as `pipelined`; 0 or 1: skip)")
    ap.add_argument("--policy-scan", action="store_true",
                    help="with --policy: the policy as a stage of its own in front of the step")
    ap.add_argument("--settle-ms", type=float, default=60.0,
                    help="keep the device busy with the calibration fill for this long before the "
                         "ticks (the clocks of an idle GPU take tens of ms to settle; untimed, and "
                         "no tick runs in it)")
    ap.add_argument("--other-workloads", type=int, default=None, metavar="TICKS",
                    help="timed ticks for each of the other workloads (c1, c2, c4, c5) reported in "
                         "`workloads` (default: 300 when the headline runs in its plain form; 0: skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (environments are independent; more GPUs "
              "would each take a slice of the env index range, no collectives). "
              "--gpus must be 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2602_01665_amd import build as hip_build
    if hip_build.is_stale():
        hip_build.build()
    from paper_2602_01665_amd import inputs as I
    from paper_2602_01665_amd.binding import TabxEnv

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    name = args.workload or I.HEADLINE
    w = I.WORKLOADS[name]
    E, N = w.num_envs, w.num_units
    over = {}
    if args.collisions or args.dynamics:
        over.update(collision_alpha=0.8)
    if args.dynamics:
        over.update(dynamics=1, move_gain=2.0, restitution=0.5)
    p = I.make_params(w, **over)
    scenario = I.make_scenario(w)
    env = TabxEnv(p, scenario, want_global_state=args.global_state)
    env.reset()
    if args.steps is None:
        args.steps = w.steps
    # one seeded action batch per tick, resident on the device before the clock starts (at most
    # 1 GiB of them; longer runs cycle)
    n_act = max(1, min(args.steps + args.warmup, (1 << 30) // (E * N)))
    if args.action_batches:
        n_act = max(1, min(n_act, args.action_batches))
    acts = [torch.from_numpy(I.actions_for_step(w.seed, s, E, N)).to("cuda:0")
            for s in range(n_act)]
    stream = torch.cuda.current_stream()
    scripted = policy = None
    if args.policy:
        policy = I.policy(args.policy, seed=w.seed)
        scripted = torch.from_numpy(np.ascontiguousarray(scenario["team"], np.uint8)).to("cuda:0")

    def tick(s):
        a = acts[s % n_act]
        if policy and args.separate:
            env.heuristic_actions(policy, scripted, a, stream)
            env.step_observe(a, stream)
        elif policy and args.policy_scan:
            env.policy_step_observe(policy, scripted, a, stream)
        elif policy:
            env.scripted_step_observe(policy, scripted, a, stream)
        elif args.separate:
            env.step(a, stream)
            env.observe(stream)
        else:
            env.step_observe(a, stream)

    if policy and not args.separate and not args.policy_scan:
        env.prime_scripted(policy, scripted, stream)
    # What a store stream can reach on this very box: a plain device fill of an obs-sized buffer
    # (always measured, before the ticks; the copy, used to scale the profiler's byte counters,
    # with --calibrate)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    # (the fill writes the observation tensor itself, which the first tick overwrites anyway)
    dst = env.obs
    nbytes = dst.numel() * 4
    cal = {"bytes": nbytes}
    jobs = [("fill", lambda: dst.fill_(1.0), nbytes)]
    if args.calibrate:
        src = torch.empty_like(env.obs)
        jobs.append(("copy", lambda: dst.copy_(src), 2 * nbytes))
    for label, fn, moved in jobs:
        t_busy = time.perf_counter()
        while True:                     # at least three, and until the device has settled
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            if label != "fill" or (time.perf_counter() - t_busy) * 1e3 >= args.settle_ms:
                break
        ev0.record(stream)
        for _ in range(20):
            fn()
        ev1.record(stream)
        torch.cuda.synchronize()
        ms = ev0.elapsed_time(ev1) / 20
        cal[label + "_ms"] = ms
        cal[label + "_GBs"] = moved / (ms * 1e-3) / 1e9

    for s in range(args.warmup):
        tick(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for s in range(args.steps):
        tick(args.warmup + s)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = ev0.elapsed_time(ev1) / args.steps     # average per tick on the launch stream
    rep_ms = [kernel_ms]
    for _ in range(max(0, args.reps - 1)):             # further repetitions, for the spread only
        ev0.record(stream)
        for s in range(args.steps):
            tick(args.warmup + s)
        ev1.record(stream)
        torch.cuda.synchronize()
        rep_ms.append(ev0.elapsed_time(ev1) / args.steps)

    assert torch.isfinite(env.obs).all()
    B_env = algorithmic_bytes_per_env(N, env.D, p["max_zones"])

    # The same batch as parts on streams of their own: one part's launch fills the start and the
    # end of another's (whole-batch throughput; the roofline above stays the single launch's).
    pipelined = None
    if args.streams > 1 and not args.separate and not args.policy_scan:
        parts = env.parts(args.streams)
        streams = [torch.cuda.Stream() for _ in parts]

        def tick_parts(s):
            a = acts[s % n_act]
            for q, st in zip(parts, streams):
                sl = slice(q.first_env, q.first_env + q.E)
                if policy:
                    q.scripted_step_observe(policy, scripted[sl], a[sl], st)
                else:
                    q.step_observe(a[sl], st)

        torch.cuda.synchronize()
        for s in range(min(args.warmup, 100)):
            tick_parts(s)
        best = None
        for _ in range(max(1, min(args.reps, 3))):
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for s in range(args.steps):
                tick_parts(args.warmup + s)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t1
            best = dt if best is None else min(best, dt)
        assert torch.isfinite(env.obs).all()
        pipelined = {"streams": len(parts), "ms_per_step": best * 1e3 / args.steps,
                     "value": E * N * args.steps / best, "unit": "agent-steps/s",
                     "algorithmic_GBs": B_env * E * args.steps / best / 1e9,
                     "frac_of_hbm_peak": B_env * E * args.steps / best / 1e9 / HBM_PEAK_GBS}

    achieved = B_env * E / (kernel_ms * 1e-3) / 1e9
    plain = not (args.collisions or args.dynamics or args.separate or args.policy or args.global_state)
    traffic, traffic_source = measured_traffic(name) if plain else (None, None)
    out = {
        "metric": "agent-steps/sec (step+observe) at 16384 envs 10v10; HBM GB/s vs peak",
        "value": E * N * args.steps / wall,
        "unit": "agent-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": name, "num_envs": E, "units_per_env": N, "obs_dim": env.D,
                   "launch": "separate step+observe" if args.separate else "fused step_observe",
                   "body_collisions": bool(args.collisions or args.dynamics),
                   "persistent_velocities": bool(args.dynamics),
                   "scripted_adversaries": args.policy,
                   "global_state_every_tick": bool(args.global_state),
                   "actions": f"{n_act} pre-generated seeded uniform action batches on the device"
                              + ("" if n_act >= args.steps + args.warmup else ", cycled")},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": B_env * E,
                     "kernel_ms": kernel_ms,
                     "kernel_ms_median": float(np.median(rep_ms)), "kernel_ms_min": min(rep_ms),
                     "repetitions": len(rep_ms)},
    }
    if pipelined:
        out["pipelined"] = pipelined
    out["calibration"] = cal
    out["roofline"]["device_fill_GBs"] = cal["fill_GBs"]
    out["roofline"]["frac_of_device_fill"] = achieved / cal["fill_GBs"]
    # the other workloads, each as its own fused tick (hipEvent-timed; the headline stays `value`)
    others = args.other_workloads if args.other_workloads is not None else (300 if plain and not args.workload else 0)
    if others > 0:
        out["workloads"] = {n: time_workload(I, TabxEnv, torch, n, min(others, I.WORKLOADS[n].steps), 50)
                            for n in ("c1_16env_3v3", "c2_4096env_5v5", "c4_65536env_5v5",
                                      "c5_1024env_64v64") if n != name}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, I, scenario, 1024 if N <= 32 else 32,
                                           1200 if N <= 32 else 300)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
