"""Helpers of the GPU parity tests: run one workload through the HIP library and
through the CPU oracle on the same arrays."""
import numpy as np
import torch

import oracle
from paper_2311_12716_amd import binding

DEV = "cuda:0"


def to_gpu(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def note(msg):
    print(f"[parity] {msg}", flush=True)


def gpu_student(w, variant=0):
    env = binding.MazeEnv(w.N, w.H, w.W, w.view, w.max_steps, device=DEV)
    env.set_kernel_variant(variant)
    env.reset_to_levels(to_gpu(w.walls), to_gpu(w.agent_xy), to_gpu(w.agent_dir), to_gpu(w.goal_xy))
    return env


def cpu_student(w):
    o = oracle.MazeOracle(w.N, w.H, w.W, w.view, w.max_steps)
    o.reset_to_levels(w.walls, w.agent_xy, w.agent_dir, w.goal_xy)
    return o


def assert_state_equal(env, o):
    xy, d, t = env.get_state()
    oxy, od, ot = o.get_state()
    assert (xy.cpu().numpy() == oxy).all(), "positions differ"
    assert (d.cpu().numpy() == od).all(), "headings differ"
    assert (t.cpu().numpy() == ot).all(), "step counters differ"


def assert_rollout_equal(gpu_out, cpu_out, what=""):
    r, d, obs = gpu_out
    orr, od, oobs = cpu_out
    d = d.cpu().numpy()
    assert (d == od).all(), f"{what}: done flags differ at {np.argwhere(d != od)[:5]}"
    r = r.cpu().numpy()
    err = np.abs(r.astype(np.float64) - orr.astype(np.float64)).max()
    assert err <= 1e-6, f"{what}: reward error {err}"
    assert ((r != 0) == (orr != 0)).all()
    if oobs is not None:
        obs = obs.cpu().numpy()
        if not (obs == oobs).all():
            bad = np.argwhere((obs != oobs).any(axis=(-1, -2, -3)))
            raise AssertionError(f"{what}: obs differ at (step, env) {bad[:5]} of {len(bad)}")


def run_fused(w, variant=0, check_state=True):
    """Whole rollout in one maze_step call vs the oracle, everything compared."""
    env, o = gpu_student(w, variant), cpu_student(w)
    obs0 = env.render_obs().cpu().numpy()
    assert (obs0 == o.render_obs()).all(), "initial observation differs"
    out = env.step(to_gpu(w.actions))
    torch.cuda.synchronize()
    ref = o.step(w.actions, w.T)
    assert_rollout_equal(out, ref, w.name)
    if check_state:
        assert_state_equal(env, o)
    return env, o, out, ref
