#!/usr/bin/env python3
"""Benchmark of the maze hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu] [--no-rows]

One "step" is one pass of the throughput workload (config 3: 32768 envs, 13x13
interior, 50 random walls, view 5, episode cap 250, 256 open-loop random actions):
maze_reset_to_levels + maze_render_obs (observation of the start state) + one
256-step maze_step launch that writes observation, reward and done for every
env-step.  Inputs are resident in HBM before the timed region.  `value` is
env-steps per second over the K timed steps.

The JSON line also carries
  roofline      achieved algorithmic HBM GB/s of the rollout kernel (81 bytes per
                env-step: 1 action in, 75 obs + 4 reward + 1 done out), timed with
                HIP events on the launch stream around every 4th maze_step of the
                timed region (an event pair costs the stream about 10 us, so not
                every pass carries one); frac_whole_pass is the same figure for the
                whole timed pass, reset and first render included;
  cpu_baseline  the CPU oracle on the same workload on this host's cores;
  rows          the other calls of the path (teacher editor at config 4, GAE,
                the 51x51 config 5 rollout, the per-step call pattern), each timed
                on its own after the main measurement.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
BYTES_PER_ENV_STEP = {5: 81, 7: 153}   # 1 action + 3k^2 obs + 4 reward + 1 done


def load_traffic():
    """HBM bytes per rollout launch measured with rocprofv3 --pmc (see profiles/)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f)
    except OSError:
        return {}


def event_ms(pairs):
    return [a.elapsed_time(b) for a, b in pairs]


def spin_up(torch, fn, ms):
    """Run fn untimed for about `ms` milliseconds of wall time; returns the number of calls.
    After an idle spell the device runs its first ~10 ms of load 5-10 % slower and unevenly
    (clock and power management settling: the editor kernel takes 145-170 us per launch for its
    first 60 launches and 145.1 from then on), which would otherwise be most of a 20-step run."""
    n = 0
    t_end = time.perf_counter() + ms * 1e-3
    while ms > 0 and time.perf_counter() < t_end:
        for _ in range(8):
            fn()
        torch.cuda.synchronize()
        n += 8
    return n


def time_calls(torch, fn, iters, warmup=2, settle_ms=20.0):
    spin_up(torch, fn, settle_ms)
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    pairs = []
    for _ in range(iters):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    ms = event_ms(pairs)
    return float(np.mean(ms)), float(np.min(ms))


def store_patterns(torch, env, actions, reward, done, obs, N, T, k):
    """The rollout's write pattern on its own (probe library), the rollout kernel and a plain
    fill, each timed over back-to-back launches; GB/s of the observation bytes written."""
    import ctypes
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2311_12716_amd", "libmaze_storeprobe.so"))
    lib.storeprobe_run.restype = ctypes.c_int
    lib.storeprobe_run.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int,
                                   ctypes.c_int, ctypes.c_void_p]
    slab = N * 3 * k * k                       # bytes per step
    groups = N // 128                          # the rollout's workgroups at 128 envs each
    obs_bytes = obs.numel()

    def probe(pattern, sleep=0):
        def fn():
            rc = lib.storeprobe_run(pattern, obs.data_ptr(), slab, groups, T, sleep,
                                    torch.cuda.current_stream().cuda_stream)
            if rc != 0:
                raise RuntimeError(f"storeprobe_run({pattern}) returned {rc}")
        return fn

    def timed(fn, iters=10):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / iters * 1e3
        return {"ms": ms, "GB/s": obs_bytes / ms / 1e6}

    spin_up(torch, lambda: obs.fill_(1), 30.0)       # settled clocks before the first pattern
    table = {"geometry": f"{groups} workgroups x {slab // groups} B per step, {T} steps, {obs_bytes} B",
             "torch_fill": timed(lambda: obs.fill_(1)),
             "probe_fill_4KB_blocks": timed(probe(0)),
             "probe_contiguous_per_workgroup": timed(probe(3)),
             "probe_slab_plain": timed(probe(1)),
             "probe_slab_plain_sleep8": timed(probe(1, 8)),
             "probe_slab_streaming": timed(probe(2))}
    for sleep in (2, 4, 6, 7, 8, 9, 10, 12, 16):
        table[f"probe_slab_streaming_sleep{sleep}"] = timed(probe(2, sleep))
    table["rollout_kernel_obs_bytes_only"] = timed(lambda: env.step(actions, reward, done, obs))
    return {"store_patterns": table}


def wave_latency(torch):
    """What one wave on an idle compute unit pays per instruction (probe library): shader clocks
    and nanoseconds per iteration of six small dependent or independent chains."""
    import ctypes
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2311_12716_amd", "libmaze_storeprobe.so"))
    lib.waveprobe_run.restype = ctypes.c_int
    lib.waveprobe_run.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    lib.waveprobe_iterations.restype = ctypes.c_int
    n = lib.waveprobe_iterations()
    out = torch.zeros(13, dtype=torch.int64, device="cuda:0")
    names = ["dependent_add", "four_independent_adds", "dependent_lds_read", "compare_select_add_chain",
             "two_compares_scalar_and_select_chain", "lds_write_then_read"]
    best = None
    for _ in range(5):          # the first launches run on clocks that have not settled
        if lib.waveprobe_run(out.data_ptr(), torch.cuda.current_stream().cuda_stream) != 0:
            raise RuntimeError("waveprobe_run failed")
        torch.cuda.synchronize()
        v = out.cpu().tolist()
        best = v if best is None or v[0] < best[0] else best
    return {"wave_latency": {name: {"clocks_per_iteration": best[2 * j] / n, "ns_per_iteration": best[2 * j + 1] / n}
                             for j, name in enumerate(names)},
            "iterations": n}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--spin-up-ms", type=float, default=50.0,
                    help="run the pass untimed for this long before the W warm-up steps, so that the "
                         "device's clocks have settled when the timed region starts (0: off)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-rows", action="store_true", help="skip the per-row measurements")
    ap.add_argument("--variant", type=int, default=0, help="0 auto, 1 per-cell kernels")
    ap.add_argument("--event-every", type=int, default=4,
                    help="bracket every n-th maze_step of the timed region with HIP events")
    ap.add_argument("--store-patterns", action="store_true",
                    help="only run the store-pattern probe (paper_2311_12716_amd/probe) at config 3's "
                         "geometry next to the rollout kernel and a plain fill, print its table")
    ap.add_argument("--wave-latency", action="store_true",
                    help="only run the single-wave latency probe (paper_2311_12716_amd/probe), print its table")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (envs are independent; sharding the batch "
              "over GPUs needs no communication and is not part of this build). Use --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2311_12716_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    binding.load_library()        # fails loudly if the HIP library is not built
    if args.wave_latency:
        print(json.dumps(wave_latency(torch)))
        return
    dev = "cuda:0"
    g = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    # ---------------------------------------------------------------- main: config 3
    w = wl.config(3)
    N, T, k = w.N, w.T, w.view
    env = binding.MazeEnv(N, w.H, w.W, k, w.max_steps, device=dev)
    env.set_kernel_variant(args.variant)
    walls, axy, adir, gxy, actions = g(w.walls), g(w.agent_xy), g(w.agent_dir), g(w.goal_xy), \
        g(w.actions)
    obs0 = torch.empty((N, k, k, 3), dtype=torch.int8, device=dev)
    reward = torch.empty((T, N), dtype=torch.float32, device=dev)
    done = torch.empty((T, N), dtype=torch.uint8, device=dev)
    obs = torch.empty((T, N, k, k, 3), dtype=torch.int8, device=dev)

    if args.store_patterns:
        print(json.dumps(store_patterns(torch, env, actions, reward, done, obs, N, T, k)))
        return

    kernel_events = []

    def one_step(record):
        env.reset_to_levels(walls, axy, adir, gxy)
        env.render_obs(obs0)
        if record:
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
        env.step(actions, reward, done, obs)
        if record:
            b.record()
            kernel_events.append((a, b))

    n_spin = spin_up(torch, lambda: one_step(False), args.spin_up_ms)
    for _ in range(args.warmup):
        one_step(False)
    torch.cuda.synchronize()
    every = max(1, args.event_every)
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(i % every == every - 1 or args.steps < every)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    env_steps = float(args.steps) * N * T
    value = env_steps / elapsed
    kms = event_ms(kernel_events)
    k_avg_s = float(np.mean(kms)) * 1e-3
    alg_bytes = BYTES_PER_ENV_STEP[k] * N * T
    achieved = alg_bytes / k_avg_s / 1e9
    # the whole pass also reads the levels (H*W wall bytes + 17 bytes of poses per env) and
    # writes the first observation
    pass_bytes = alg_bytes + N * (w.H * w.W + 17) + N * 3 * k * k
    pass_gbs = pass_bytes / (elapsed / args.steps) / 1e9
    traffic = load_traffic().get("student_rollout_c3")
    n_resets = int(done.sum().item())

    out = {
        "metric": "env-steps/sec (student maze step + obs render)",
        "value": value,
        "unit": "env-steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "spin_up": {"ms": args.spin_up_ms, "untimed_passes": n_spin,
                    "what": "the same pass run untimed before the W warm-up steps until the device's "
                            "clocks have settled after idling; --spin-up-ms 0 turns it off"},
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32 bit-packed grids / int8 obs / f32 reward",
        "data": "synthetic",
        "config": {"workload": w.name, "envs": N, "grid": "13x13", "walls": 50, "view": k,
                   "max_steps": w.max_steps, "rollout_steps": T, "resets_per_rollout": n_resets,
                   "kernel_variant": args.variant},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "student rollout (maze_step, 256 steps fused)",
                     "kernel_ms_avg": k_avg_s * 1e3, "kernel_ms_min": float(np.min(kms)),
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "timing": f"HIP events on the launch stream around {len(kms)} of the {args.steps} "
                               "timed maze_step launches; bytes are algorithmic, `traffic` is the "
                               "counter figure of profiles/hbm_traffic.json",
                     "frac_whole_pass": pass_gbs / HBM_PEAK_GBS,
                     "whole_pass": {"achieved": pass_gbs, "algorithmic_bytes": pass_bytes,
                                    "ms": elapsed / args.steps * 1e3,
                                    "what": "reset to levels + first render + rollout, wall clock "
                                            "over the timed region"}},
    }

    if args.calib_copy:
        # a plain copy of known size: 256 MiB read + 256 MiB written per launch
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------------------------------------------------------- other rows
    if not args.no_rows:
        rows = {}
        ms, mn = time_calls(torch, lambda: env.reset_to_levels(walls, axy, adir, gxy), 20)
        rows["maze_reset_to_levels_c3"] = {"ms": ms, "GB/s": N * (169 + 17) / ms / 1e6}
        ms, mn = time_calls(torch, lambda: env.render_obs(obs0), 20)
        rows["maze_render_obs_c3"] = {"ms": ms, "GB/s": N * 75 / ms / 1e6}
        # where the time of a pass goes: each call alone, launches back to back, and the rest
        ms_roll, mn = time_calls(torch, lambda: env.step(actions, reward, done, obs), 20, warmup=3)
        rows["pass_breakdown_c3"] = {
            "pass_ms": out["ms_per_step"], "rollout_ms": ms_roll,
            "reset_plus_render_ms": out["ms_per_step"] - ms_roll,
            "note": "rollout = maze_step alone, launches back to back; the rest is what reset to levels "
                    "and the first render add to a pass (their kernels, the gaps between three dependent "
                    "launches, the packing kernel running behind the rollout's last writes); kernel by "
                    "kernel: profiles/kernels.md"}
        # the same pass replayed from a captured HIP graph
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            one_step(False)
        torch.cuda.current_stream().wait_stream(side)
        pass_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(pass_graph):
            one_step(False)
        for _ in range(3):
            pass_graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(30):
            pass_graph.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - g0) / 30 * 1e3
        rows["pass_graph_replay_c3"] = {"ms": g_ms, "env-steps/s": N * T / g_ms * 1e3,
                                        "note": "reset + render + rollout captured once, replayed 30 times"}
        del pass_graph
        a1 = actions[:1].contiguous()
        r1, d1 = reward[:1], done[:1]

        def per_step():
            env.step(a1, r1, d1, None, want_obs=False)
            env.render_obs(obs0)
        ms, mn = time_calls(torch, per_step, 200, warmup=20)
        rows["per_step_call_pattern_c3"] = {"ms": ms, "env-steps/s": N / ms * 1e3,
                                            "note": "maze_step(n=1) + maze_render_obs, launch-bound"}
        nwalls = torch.empty((N,), dtype=torch.int32, device=dev)
        plen = torch.empty((N,), dtype=torch.int32, device=dev)
        ms, mn = time_calls(torch, lambda: env.level_metrics(nwalls, plen), 50)
        rows["maze_level_metrics_c3"] = {"ms": ms, "levels/s": N / ms * 1e3,
                                         "note": "wall count + shortest path (bit-parallel flood)"}
        o1 = obs[:1]
        ms, mn = time_calls(torch, lambda: env.step(a1, r1, d1, o1), 200, warmup=20)
        rows["per_step_with_obs_c3"] = {"ms": ms, "env-steps/s": N / ms * 1e3,
                                        "note": "maze_step(n=1) writing obs: one launch per step"}
        # observation variants (occluded view, type/colour/state bytes)
        env.set_obs_mode(1, 1)
        ms, mn = time_calls(torch, lambda: env.step(actions, reward, done, obs), 30, warmup=30)
        rows["student_rollout_c3_occluded_typed_obs"] = {
            "ms": ms, "env-steps/s": N * T / ms * 1e3, "GB/s": 81.0 * N * T / ms / 1e6,
            "note": "maze_set_obs_mode(1, 1): occlusion in the records stage, typed bytes in the store stage"}
        for mode, name in (((1, 0), "typed_obs"), ((0, 1), "occluded_obs")):
            env.set_obs_mode(*mode)
            ms, mn = time_calls(torch, lambda: env.step(actions, reward, done, obs), 30, warmup=30)
            rows["student_rollout_c3_" + name] = {
                "ms": ms, "env-steps/s": N * T / ms * 1e3, "GB/s": 81.0 * N * T / ms / 1e6,
                "note": "maze_set_obs_mode(%d, %d)" % mode}
        env.set_obs_mode(0, 0)
        # the same single step replayed from a captured HIP graph (what a policy loop can do)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            env.step(a1, r1, d1, o1)
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(16):
                env.step(a1, r1, d1, o1)
        ms, mn = time_calls(torch, graph.replay, 50, warmup=5)
        rows["per_step_with_obs_graph16_c3"] = {"ms": ms / 16, "env-steps/s": 16 * N / ms * 1e3,
                                                "note": "16 single steps per captured graph replay"}
        del graph
        # closed-loop stepping at the batch sizes of the paper's speed table (Section 3, steps
        # per second at 1 / 32 / 256 / 1024 parallel envs): one maze_step(n=1) with obs per step
        small = {}
        for Ns in (1, 32, 256, 1024):
            ws = wl.student_random(f"table-{Ns}", 900 + Ns, N=Ns, T=4, n_walls=50)
            es = binding.MazeEnv(Ns, ws.H, ws.W, ws.view, ws.max_steps, device=dev)
            es.reset_to_levels(g(ws.walls), g(ws.agent_xy), g(ws.agent_dir), g(ws.goal_xy))
            a_s = g(ws.actions[:1])
            r_s = torch.empty((1, Ns), dtype=torch.float32, device=dev)
            d_s = torch.empty((1, Ns), dtype=torch.uint8, device=dev)
            o_s = torch.empty((1, Ns, 5, 5, 3), dtype=torch.int8, device=dev)
            ms, mn = time_calls(torch, lambda: es.step(a_s, r_s, d_s, o_s), 200, warmup=20)
            small[str(Ns)] = {"ms": ms, "env-steps/s": Ns / ms * 1e3}
            del es
        rows["closed_loop_single_steps_by_batch"] = small
        # GAE on this rollout's outputs
        values = torch.rand((T + 1, N), dtype=torch.float32, device=dev)
        adv = torch.empty((T, N), dtype=torch.float32, device=dev)
        ret = torch.empty((T, N), dtype=torch.float32, device=dev)
        ms, mn = time_calls(torch, lambda: binding.compute_gae(reward, values, done, 0.995, 0.98,
                                                               adv, ret), 20)
        rows["compute_gae_T256_N32768"] = {"ms": ms, "GB/s": 17.0 * N * T / ms / 1e6}
        ms, mn = time_calls(torch, lambda: binding.replay_scores(reward, values, done, adv, 0.995), 20)
        rows["replay_scores_T256_N32768"] = {"ms": ms, "GB/s": 13.0 * N * T / ms / 1e6,
                                             "note": "best return, MaxMC, PVL per level; reads 13 B per env-step"}
        # replay distribution over a buffer of the paper's size
        Kb = 4000
        sc = torch.rand((Kb,), device=dev)
        seen = torch.randint(0, 1000, (Kb,), dtype=torch.int32, device=dev)
        pb = torch.empty((Kb,), dtype=torch.float32, device=dev)
        ms, mn = time_calls(torch, lambda: binding.replay_distribution(sc, seen, 1000, True, 0.3, 0.3, pb), 50)
        rows["replay_distribution_K4000_rank"] = {"ms": ms, "note": "one workgroup: bitonic sort in LDS, two block sums"}
        del values, adv, ret
        # config 2 sized GAE
        N2, T2 = 4096, 256
        r2 = torch.rand((T2, N2), device=dev)
        v2 = torch.rand((T2 + 1, N2), device=dev)
        d2 = (torch.rand((T2, N2), device=dev) < 0.01).to(torch.uint8)
        a2, rt2 = torch.empty_like(r2), torch.empty_like(r2)
        ms, mn = time_calls(torch, lambda: binding.compute_gae(r2, v2, d2, 0.995, 0.98, a2, rt2), 50)
        rows["compute_gae_c2_T256_N4096"] = {"ms": ms, "GB/s": 17.0 * N2 * T2 / ms / 1e6}
        # teacher editor, config 4
        ew = wl.config(4)
        ed = binding.EditorEnv(ew.N, ew.H, ew.W, ew.n_walls, device=dev)
        eact, edir = g(ew.actions), g(ew.agent_dir_init)
        eobs = torch.empty((ew.T, ew.N, ew.H, ew.W, 3), dtype=torch.int8, device=dev)
        et = torch.empty((ew.T, ew.N), dtype=torch.int32, device=dev)
        edn = torch.empty((ew.T, ew.N), dtype=torch.uint8, device=dev)

        def editor_pass():
            ed.reset(edir)
            ed.step(eact, eobs, et, edn)
        ms, mn = time_calls(torch, editor_pass, 30, warmup=30)
        ebytes = 516.0 * ew.N * ew.T   # 4 action + 507 obs + 4 t + 1 done
        rows["editor_c4"] = {"ms": ms, "editor-steps/s": ew.N * ew.T / ms * 1e3,
                             "GB/s": ebytes / ms / 1e6, "frac_of_hbm_peak": ebytes / ms / 1e6 / HBM_PEAK_GBS}
        ms, mn = time_calls(torch, lambda: ed.random_levels(1, 0), 20)
        rows["editor_random_levels_c4"] = {"ms": ms, "levels/s": ew.N / ms * 1e3,
                                           "note": "52 placements per level from the counter-based generator"}
        ms, mn = time_calls(torch, lambda: ed.mutate_levels(2, 0, 20), 20)
        rows["editor_mutate_levels_c4_20edits"] = {"ms": ms, "levels/s": ew.N / ms * 1e3}
        del eobs, et, edn, ed
        # configs 1 and 2: small batches (latency-bound)
        for ci in (1, 2):
            wc = wl.config(ci)
            ec = binding.MazeEnv(wc.N, wc.H, wc.W, wc.view, wc.max_steps, device=dev)
            ec.reset_to_levels(g(wc.walls), g(wc.agent_xy), g(wc.agent_dir), g(wc.goal_xy))
            ac = g(wc.actions)
            rc_ = torch.empty((wc.T, wc.N), dtype=torch.float32, device=dev)
            dc = torch.empty((wc.T, wc.N), dtype=torch.uint8, device=dev)
            oc = torch.empty((wc.T, wc.N, 5, 5, 3), dtype=torch.int8, device=dev)
            ms, mn = time_calls(torch, lambda: ec.step(ac, rc_, dc, oc), 20)
            rows[f"student_rollout_c{ci}"] = {"ms": ms, "env-steps/s": wc.N * wc.T / ms * 1e3,
                                              "GB/s": 81.0 * wc.N * wc.T / ms / 1e6}
            del ec, oc
        # config 5: 51x51 perfect mazes, view 7
        w5 = wl.config(5)
        env5 = binding.MazeEnv(w5.N, w5.H, w5.W, w5.view, w5.max_steps, device=dev)
        env5.set_kernel_variant(args.variant)
        env5.reset_to_levels(g(w5.walls), g(w5.agent_xy), g(w5.agent_dir), g(w5.goal_xy))
        a5 = g(w5.actions)
        r5 = torch.empty((w5.T, w5.N), dtype=torch.float32, device=dev)
        d5 = torch.empty((w5.T, w5.N), dtype=torch.uint8, device=dev)
        o5 = torch.empty((w5.T, w5.N, 7, 7, 3), dtype=torch.int8, device=dev)
        ms, mn = time_calls(torch, lambda: env5.step(a5, r5, d5, o5), 30, warmup=30)
        b5 = 153.0 * w5.N * w5.T
        rows["student_rollout_c5"] = {"ms": ms, "env-steps/s": w5.N * w5.T / ms * 1e3,
                                      "GB/s": b5 / ms / 1e6, "frac_of_hbm_peak": b5 / ms / 1e6 / HBM_PEAK_GBS}
        env5.set_obs_mode(0, 1)
        ms, mn = time_calls(torch, lambda: env5.step(a5, r5, d5, o5), 30, warmup=30)
        rows["student_rollout_c5_occluded_obs"] = {"ms": ms, "env-steps/s": w5.N * w5.T / ms * 1e3,
                                                   "GB/s": b5 / ms / 1e6,
                                                   "frac_of_hbm_peak": b5 / ms / 1e6 / HBM_PEAK_GBS,
                                                   "note": "maze_set_obs_mode(0, 1) on config 5"}
        env5.set_obs_mode(0, 0)
        nw5 = torch.empty((w5.N,), dtype=torch.int32, device=dev)
        pl5 = torch.empty((w5.N,), dtype=torch.int32, device=dev)
        ms, mn = time_calls(torch, lambda: env5.level_metrics(nw5, pl5), 20)
        rows["maze_level_metrics_c5"] = {"ms": ms, "levels/s": w5.N / ms * 1e3,
                                         "mean_path_len": float(pl5.float().mean())}
        del o5, env5
        # plain streaming-write ceiling of this GPU (torch fill of the obs buffer)
        ms, mn = time_calls(torch, lambda: obs.fill_(1), 10)
        rows["fill_ceiling"] = {"ms": ms, "GB/s": obs.numel() / ms / 1e6,
                                "note": "torch fill_ of the 629 MB obs tensor"}
        out["rows"] = rows

    # ---------------------------------------------------------------- CPU oracle
    if not args.no_cpu:
        import oracle
        o = oracle.MazeOracle(N, w.H, w.W, k, w.max_steps)
        cpu_steps, t_cpu = 0, 0.0
        reps = 0
        while t_cpu < 10.0 and reps < 1000:
            o.reset_to_levels(w.walls, w.agent_xy, w.agent_dir, w.goal_xy)
            c0 = time.perf_counter()
            o.render_obs()
            o.step(w.actions, T)
            t_cpu += time.perf_counter() - c0
            cpu_steps += N * T
            reps += 1
        out["cpu_baseline"] = {"value": cpu_steps / t_cpu, "unit": "env-steps/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"{reps} x the full config-3 rollout "
                                         f"({N} envs x {T} steps, step + render), {t_cpu:.1f} s"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
