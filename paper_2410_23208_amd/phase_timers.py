#!/usr/bin/env python3
"""Where the step kernel spends its clocks: runs a workload on the instrumented build of the library
(-DK2D_PHASE_TIMERS, built on the spot as libk2d_timers.so) and prints, per phase of a substep, the share of
the wavefronts' clocks and the clocks per wavefront-substep -- for all wavefronts, for the slowest eight (the
ones a launch of resident wavefronts waits for) and for the median eight.

  python -m paper_2410_23208_amd.phase_timers [--config 2] [--envs N] [--steps K] [--no-build] [--alone]
                                              [--sweep-order tournament|levels]

--alone: every environment of the workload in a wavefront of its own (three empty environments beside it, the
ordering of the launch switched off), 2048 at a time: how long the chain of one environment is by itself --
what a launch of resident wavefronts cannot be shorter than.
"""
import argparse
import ctypes
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

PHASES = ["actions", "gravity + world polygons", "joint constants", "motors + thrusters", "cull + candidate list",
          "manifolds", "take + pre-solve", "levels of the pairs", "warm start", "sweeps: joints", "sweeps: collisions",
          "Euler step", "corrections: collisions", "corrections: joints", "restarts / tail"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--envs", type=int, default=0)
    ap.add_argument("--steps", type=int, default=0)
    ap.add_argument("--no-build", action="store_true", help="use the libk2d_timers.so that is there")
    ap.add_argument("--alone", action="store_true", help="one environment per wavefront (see above)")
    ap.add_argument("--sweep-order", default="tournament", choices=["tournament", "levels"],
                    help="visiting order of the colliding pairs (k2d_params.sweep_order)")
    args = ap.parse_args()
    import torch          # first: the library must bind to the HIP runtime that torch has loaded
    import scenegen
    from paper_2410_23208_amd import build as hip_build, binding
    path = hip_build.LIB_TIMERS if args.no_build else hip_build.build(phase_timers=True)
    L = binding.use_library(path)
    L.k2d_debug_set_phase_buffer.argtypes = [ctypes.c_void_p, ctypes.c_long]
    import paper_2410_23208_amd as k2d
    cfg = scenegen.CONFIGS[args.config]
    n_envs = args.envs or cfg["n_envs"]
    n_steps = args.steps or cfg["n_steps"]
    caps, params, scene = scenegen.make_scene(args.config, n_envs=n_envs)
    params = dict(params, sweep_order=1 if args.sweep_order == "levels" else 0)
    act = torch.from_numpy(scenegen.make_actions(args.config, n_steps, n_envs)).cuda()
    words = torch.from_numpy(k2d.pack_scenes(caps, scene).view(np.int32)).cuda()
    if args.alone:
        return alone(L, k2d, torch, scenegen, caps, params, scene, scenegen.make_actions(args.config, n_steps, n_envs),
                     n_envs, n_steps, cfg)
    n_waves = (n_envs + 3) // 4
    slots = L.k2d_debug_set_phase_buffer(None, 0)
    buf = torch.zeros((n_waves, slots), dtype=torch.int64, device="cuda")
    L.k2d_debug_set_phase_buffer(buf.data_ptr(), n_waves)
    b = k2d.Batch(caps, n_envs, params)
    for rep in range(2):
        b.reset(words)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        b.step(act, n_steps)
        e1.record()
        torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    v = buf.cpu().numpy().astype(np.float64)
    ph, lv = v[:, :len(PHASES)], v[:, len(PHASES):]
    tot = ph.sum(1)
    nsub = n_steps * params["n_substeps"]
    print("workload %d (%s): %d environments x %d steps, %d wavefronts; instrumented launch %.2f ms"
          % (args.config, cfg["name"], n_envs, n_steps, n_waves, ms))
    print("clocks per wavefront: mean %.1fM  p50 %.1fM  p90 %.1fM  p99 %.1fM  max %.1fM  min %.1fM"
          % tuple(x / 1e6 for x in (tot.mean(), np.percentile(tot, 50), np.percentile(tot, 90), np.percentile(tot, 99),
                                    tot.max(), tot.min())))
    order = np.argsort(-tot)
    for tag, sel in (("all wavefronts", order), ("slowest 8", order[:8]), ("median 8", order[n_waves // 2 - 4:n_waves // 2 + 4])):
        sel = sel[:max(1, len(sel))]
        print("%s: %.1fM clocks, %.0f per substep; collision levels per substep %.2f, joint levels %.2f"
              % (tag, tot[sel].mean() / 1e6, tot[sel].mean() / nsub, lv[sel, 0].mean() / nsub, lv[sel, 1].mean() / nsub))
        for name, x in zip(PHASES, ph[sel].mean(0)):
            print("   %-26s %5.1f %%  %8.0f clocks per wavefront-substep" % (name, 100.0 * x / tot[sel].mean(), x / nsub))
    L.k2d_debug_set_phase_buffer(None, 0)


def alone(L, k2d, torch, scenegen, caps, params, scene, act, n_envs, n_steps, cfg):
    L.k2d_debug_keep_order(1)
    slots = L.k2d_debug_set_phase_buffer(None, 0)
    nsub = n_steps * params["n_substeps"]
    tot, ids, phases, levels = [], [], [], []
    for lo in range(0, n_envs, 2048):
        envs = np.arange(lo, min(lo + 2048, n_envs))
        order = np.repeat(envs, 4)
        empty = np.nonzero(np.arange(len(order)) % 4 != 0)[0]
        sc = scenegen.select_envs(scene, order)
        for name in ("active", "joint_active", "thruster_active"):
            sc[name] = sc[name].copy()
            sc[name][empty] = 0
        words = torch.from_numpy(k2d.pack_scenes(caps, sc).view(np.int32)).cuda()
        a = torch.from_numpy(np.ascontiguousarray(act[:, order])).cuda()
        buf = torch.zeros((len(envs), slots), dtype=torch.int64, device="cuda")
        L.k2d_debug_set_phase_buffer(buf.data_ptr(), len(envs))
        b = k2d.Batch(caps, len(order), params)
        b.reset(words)
        b.step(a, n_steps)
        torch.cuda.synchronize()
        v = buf.cpu().numpy().astype(np.float64)
        L.k2d_debug_set_phase_buffer(None, 0)
        tot.append(v[:, :len(PHASES)].sum(1)); ids.append(envs); phases.append(v[:, :len(PHASES)]); levels.append(v[:, len(PHASES):])
    L.k2d_debug_keep_order(0)
    tot, ids, phases, levels = np.concatenate(tot), np.concatenate(ids), np.concatenate(phases), np.concatenate(levels)
    print("workload (%s): %d environments x %d steps, one environment per wavefront" % (cfg["name"], n_envs, n_steps))
    print("clocks per environment: mean %.1fM  p50 %.1fM  p90 %.1fM  p99 %.1fM  max %.1fM  min %.1fM"
          % tuple(x / 1e6 for x in (tot.mean(), np.percentile(tot, 50), np.percentile(tot, 90), np.percentile(tot, 99),
                                    tot.max(), tot.min())))
    for w in np.argsort(-tot)[:8]:
        print("environment %5d: %.1fM clocks, %.0f per substep; collision levels per substep %.2f, joint levels %.2f; "
              "sweeps %.0f + %.0f, manifolds %.0f, everything else %.0f clocks per substep"
              % (ids[w], tot[w] / 1e6, tot[w] / nsub, levels[w, 0] / nsub, levels[w, 1] / nsub, phases[w, 10] / nsub,
                 phases[w, 9] / nsub, phases[w, 5] / nsub, (tot[w] - phases[w, 10] - phases[w, 9] - phases[w, 5]) / nsub))


if __name__ == "__main__":
    main()
