#!/usr/bin/env python3
"""Throughput of the batched 2D rigid-body step on one MI355X.

One "step" of this benchmark is one pass of the whole hot path over one batch: `k2d_step` advancing every
environment of the workload by its full number of engine steps (config "L": 8192 environments x 256
steps, 3 substeps x 10 solver sweeps), starting from the freshly reset synthetic scenes.  Inputs (scenes,
actions) are resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 0..4] [--workload config|dense|towers]
                  [--batch-size B] [--sweep-order tournament|levels] [--cpu-envs N] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

FP32_VALU_PEAK_TFLOPS = 157.3   # MI355X vector fp32: 256 CU x 4 SIMD x 16 lanes x 2 (packed) x 2 (fma) x 2.4 GHz
FP32_VALU_PEAK_NONPACKED = 78.6 # the same without packed fp32 instructions (this build issues none)
CLOCK_GHZ = 2.4


def read_traffic(name):
    """(HBM bytes per launch, commit the counters were collected at) from the committed rocprofv3 counter
    summary of this workload; (None, None) if there is none."""
    path = os.path.join(ROOT, "profiles", "k2d_step_%s_hbm_traffic.txt" % name)
    val, at = None, None
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch="):
                    val = float(line.split("=", 1)[1])
                if line.startswith("profiled_at_commit="):
                    at = line.split("=", 1)[1].strip()
    except OSError:
        pass
    return val, at


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=2, help="workload 0..4 (default 2 = L, 8192 envs x 256 steps)")
    ap.add_argument("--workload", default="config", choices=["config", "dense", "towers"],
                    help="config = the workload --config names; dense = workload 3's heap in a narrow pen "
                         "(contact-heavy), towers = stacks of boxes (A.7); both 8192 environments x 256 steps")
    ap.add_argument("--cpu-envs", type=int, default=8192, help="environments of the CPU-oracle sample")
    ap.add_argument("--batch-size", type=int, default=0, help="0 = the default schedule (levels of independent constraints: a "
                    "sequential sweep's bits); 1..32 = the batched impulse resolution of A.8 with that batch size")
    ap.add_argument("--sweep-order", default="tournament", choices=["tournament", "levels"],
                    help="visiting order of the colliding pairs in a sweep (k2d_params.sweep_order): the order of "
                    "a round-robin tournament over the shapes (default), or level after level (lowest free level)")
    ap.add_argument("--calibrate-copy", action="store_true", help="also run one plain 256 MiB device copy, so "
                    "that a counter run has a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg (flop model then uses "
                    "a 256-environment oracle run only for the contact statistics)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (environments are independent; more GPUs would each take "
              "a slice of the environment axis with no exchange); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import torch
    import scenegen
    import paper_2410_23208_amd as k2d
    from paper_2410_23208_amd import workmodel

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    if args.workload == "config":
        cfg = scenegen.CONFIGS[args.config]
        n_envs, n_steps = cfg["n_envs"], cfg["n_steps"]
        caps, params, scene = scenegen.make_scene(args.config)
        actions_h = scenegen.make_actions(args.config, n_steps, n_envs)
        wl_name = "config %d: %s" % (args.config, cfg["name"])
    else:
        n_envs, n_steps = 8192, 256
        if args.workload == "dense":
            caps, params, scene = scenegen.make_dense_scene(n_envs=n_envs)
            actions_h = scenegen.make_actions(3, n_steps, n_envs)
        else:
            caps, params, scene = scenegen.make_stack_scene(n_envs=n_envs)
            actions_h = np.zeros((n_steps, n_envs, caps[2] + caps[3]), dtype=np.float32)
        cfg = dict(name=args.workload)
        wl_name = {"dense": "dense pile (workload 3's generator in a 1.8 m pen)", "towers": "towers of boxes (A.7)"}[args.workload]
    params = dict(params, batch_size=args.batch_size, sweep_order=1 if args.sweep_order == "levels" else 0)
    dev = torch.device("cuda:0")
    words = torch.from_numpy(k2d.pack_scenes(caps, scene).view(np.int32)).to(dev)
    actions = torch.from_numpy(actions_h).to(dev)
    batch = k2d.Batch(caps, n_envs, params)
    # workload 4: after every step a seeded 5 % of the environments start a new episode (inside the launch,
    # from a device-resident pool that holds one fresh scene per environment)
    restarts = args.workload == "config" and args.config == 4
    if restarts:
        _, _, fresh = scenegen.make_scene(args.config, episode=1)
        pool = torch.from_numpy(k2d.pack_scenes(caps, fresh).view(np.int32)).to(dev)
        sched_h = np.full((n_steps, n_envs), -1, dtype=np.int32)
        for s in range(n_steps):
            ids = scenegen.reset_ids(args.config, s, n_envs)
            sched_h[s, ids] = ids
        sched = torch.from_numpy(sched_h).to(dev)
    torch.cuda.synchronize()

    def one_pass(ev=None):
        batch.reset(words)
        if ev:
            ev[0].record()
        if restarts:
            batch.step_reset(actions, pool, sched, n_steps)
        else:
            batch.step(actions, n_steps)
        if ev:
            ev[1].record()

    if args.calibrate_copy:
        src = torch.empty(64 << 20, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        one_pass()
    torch.cuda.synchronize()
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_pass(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = [a.elapsed_time(b) for a, b in events]
    env_steps = n_envs * n_steps
    value = args.steps * env_steps / wall

    # ---- CPU oracle on a bounded sample of the same workload: baseline + contact statistics ----
    from oracle.k2d_oracle import Oracle
    cores = min(len(os.sched_getaffinity(0)), 16)
    ns = min(n_envs, 256 if args.no_cpu else args.cpu_envs)
    sub = scenegen.select_envs(scene, np.arange(ns))
    ora = Oracle(caps, ns, params, "f32")
    ora.load_scene(sub)
    t1 = time.perf_counter()
    if restarts:
        for s in range(n_steps):
            ora.step(actions_h[s:s + 1, :ns], n_threads=cores)
            ids = scenegen.reset_ids(args.config, s, n_envs)
            ids = ids[ids < ns]
            if len(ids):
                ora.load_scene(scenegen.select_envs(fresh, ids), env_ids=ids)
    else:
        ora.step(actions_h[:, :ns], n_threads=cores)
    cpu_t = time.perf_counter() - t1
    nsub = ora.get("substeps_done").sum()
    slots = ora.get("active_slots_sum").sum() / nsub
    pairs = ora.get("active_pairs_sum").sum() / nsub
    ppov = ora.get("pp_overlap_sum").sum() / nsub
    flops_step, st = workmodel.flops_per_env_step(caps, scene, params, slots, pairs, ppov)

    # two figures from states sampled along a small CPU run of the same scenes (no restarts): the arithmetic
    # of the manifolds the kernel really evaluates (bounding-box survivors), and the chain of constraint
    # visits that the sweep order forces to run one after the other in the heaviest sampled environment
    from oracle.k2d_oracle import schedule
    n_s = min(ns, 128)
    N_sh = caps[0] + caps[1]
    sub_s = scenegen.select_envs(scene, np.arange(n_s))
    ora_s = Oracle(caps, n_s, params, "f32")
    ora_s.load_scene(sub_s)
    sa, sb, _ = schedule(N_sh)
    every = max(1, n_steps // 16)
    f_exec, chain = [], np.zeros(n_s)
    for s0 in range(0, n_steps, every):
        s1 = min(n_steps, s0 + every)
        ora_s.step(actions_h[s0:s1, :n_s], n_threads=cores)
        st_s = ora_s.state()
        f_exec.append(workmodel.executed_manifold_flops(caps, sub_s, st_s["pos"].reshape(n_s, N_sh, 2), st_s["theta"])[0])
        chain += workmodel.sequential_chain_instructions(caps, sub_s, params, st_s["pair_count"], (sa, sb)) \
            * (s1 - s0) * params["n_substeps"]
    flops_exec = flops_step - params["n_substeps"] * (st["f_manifolds"] - float(np.mean(f_exec)))
    chain_bound_ms = float(chain.max()) * 4.0 / (CLOCK_GHZ * 1e6)

    # spot check of the timed path against the oracle (same launch configuration, sampled environments)
    gs = k2d.unpack_state(caps, batch.read_state()[:ns].cpu().numpy())
    os_ = ora.state()
    parity_ok = all(np.array_equal(gs[k], os_[k]) for k in ("pos", "theta", "vel", "omega", "pair_count"))

    kern_avg = float(np.mean(kern_ms)) * 1e-3
    achieved = flops_step * env_steps / kern_avg / 1e12
    executed = flops_exec * env_steps / kern_avg / 1e12
    traffic, traffic_at = read_traffic(cfg["name"]) if (args.batch_size == 0 and args.workload == "config"
                                                              and args.sweep_order == "tournament") else (None, None)
    out = {
        "metric": "physics env-steps/sec on 1 MI355X (%s scenes, %d envs)" % (cfg["name"], n_envs),
        "value": value, "unit": "env-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s, %d envs x %d steps, %d substeps x %d solver sweeps, caps P/C/J/T=%s"
                   % (wl_name, n_envs, n_steps, params["n_substeps"], params["n_iters"], "/".join(map(str, caps))),
                   "env_steps_per_launch": env_steps, "seed": scenegen.SEED,
                   "schedule": ("sequential sweep, %s" % ("level after level" if args.sweep_order == "levels"
                                                         else "tournament order")) if args.batch_size == 0
                   else "batches of %d (A.8)" % args.batch_size},
        "roofline": {"bound": "alu", "achieved": achieved, "peak": FP32_VALU_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / FP32_VALU_PEAK_TFLOPS, "traffic": traffic, "traffic_profiled_at": traffic_at,
                     "frac_nonpacked": achieved / FP32_VALU_PEAK_NONPACKED,
                     "flops_executed_per_env_step": flops_exec, "frac_executed": executed / FP32_VALU_PEAK_TFLOPS,
                     "chain_bound_ms": chain_bound_ms,
                     "chain_bound_note": "constraint visits that the sweep order forces to run one after the other in "
                                         "the heaviest of %d sampled environments, 54 instructions per manifold point "
                                         "and 31 (+8) per joint, one instruction per 4 clocks at %.1f GHz" % (n_s, CLOCK_GHZ),
                     "kernel": "k2d_step_kernel", "kernel_ms_avg": kern_avg * 1e3, "kernel_ms": kern_ms,
                     "flops_per_env_step": flops_step, "active_points_per_substep": float(slots),
                     "active_pairs_per_substep": float(pairs), "eligible_pairs": st["n_eligible"],
                     "hbm_GBps_algorithmic": (2 * 4 * k2d.get_layout(caps)["state_words"] * n_envs
                                              + 4 * actions.numel()) / kern_avg / 1e9},
        "cpu_baseline": {"value": ns * n_steps / cpu_t, "unit": "env-steps/s", "cores": cores, "kind": "oracle",
                         "sample": "first %d of %d environments, all %d steps, fp32 oracle, %d threads, %.1f s"
                                   % (ns, n_envs, n_steps, cores, cpu_t)},
        "parity_spot_check": "bit-identical to the oracle on %d sampled environments" % ns if parity_ok
                             else "MISMATCH against the oracle on the sampled environments",
    }
    print(json.dumps(out))
    if not parity_ok:
        sys.exit(1)


if __name__ == "__main__":
    main()
