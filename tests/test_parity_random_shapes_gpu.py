"""GPU parity on shapes drawn at random (seeded): grid sizes, view sizes, batch sizes, rollout
lengths, episode caps and observation modes that no hand-picked case fixes, each compared with
the oracle byte for byte through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_12716_amd import binding, workloads as wl
from parity_util import (DEV, assert_rollout_equal, assert_state_equal, cpu_student, gpu_student, note,
                         to_gpu)

pytestmark = pytest.mark.gpu


def _student_case(seed):
    rng = np.random.default_rng(seed)
    H, W = int(rng.integers(1, 41)), int(rng.integers(1, 41))
    if H * W < 2:
        W = 2
    k = int(rng.choice([3, 5, 7, 9]))
    N = int(rng.choice([1, 31, 32, 33, 64, 96, 130, 257, 500]))
    T = int(rng.integers(1, 70))
    max_steps = int(rng.choice([1, 2, 7, 40, 250]))
    n_walls = int(rng.integers(0, max(1, H * W - 1)))
    mode = (int(rng.integers(0, 2)), int(rng.integers(0, 2)))
    return H, W, k, N, T, max_steps, n_walls, mode


@pytest.mark.parametrize("seed", range(4000, 4032))
def test_student_random_shape(seed):
    H, W, k, N, T, max_steps, n_walls, mode = _student_case(seed)
    w = wl.student_random(f"random-shape-{seed}", seed, N=N, H=H, W=W, view=k, T=T, n_walls=n_walls,
                          max_steps=max_steps)
    note(f"{w.name}: N={N} {H}x{W} k={k} T={T} max_steps={max_steps} walls={n_walls} mode={mode}")
    env, o = gpu_student(w), cpu_student(w)
    env.set_obs_mode(*mode)
    o.set_obs_mode(*mode)
    assert (env.render_obs().cpu().numpy() == o.render_obs()).all(), "initial observation differs"
    # the rollout in two calls (state carried), then one more single step
    cut = T // 2
    acts = to_gpu(w.actions)
    outs = [env.step(acts[:cut])] if cut else []
    outs.append(env.step(acts[cut:]))
    torch.cuda.synchronize()
    r = torch.cat([x[0] for x in outs]); d = torch.cat([x[1] for x in outs]); obs = torch.cat([x[2] for x in outs])
    ref = o.step(w.actions, T)
    assert_rollout_equal((r, d, obs), ref, w.name)
    assert_state_equal(env, o)
    n_walls_gpu, path_gpu = env.level_metrics()
    onw, opl = oracle.level_metrics(w.walls, w.agent_xy, w.goal_xy)
    assert (n_walls_gpu.cpu().numpy() == onw).all() and (path_gpu.cpu().numpy() == opl).all()


@pytest.mark.parametrize("seed", range(4500, 4516))
def test_student_random_shape_large_batches(seed):
    """The same with batch sizes around the limits at which the launcher changes the workgroup
    size (16, 32, 64, 128 envs), odd action bytes among the actions, and the rollout cut in two at
    a random step."""
    rng = np.random.default_rng(seed)
    k = int(rng.choice([3, 5, 7]))
    H, W = int(rng.integers(2, 30)), int(rng.integers(2, 30))
    N = int(rng.choice([4095, 4096, 4097, 4200, 8191, 8208, 16383, 16384, 16400, 32767, 32768, 33000]))
    T = int(rng.choice([7, 9, 17, 33, 65, 66]))
    max_steps = int(rng.choice([1, 3, 11, 50]))
    n_walls = int(rng.integers(0, H * W - 1))
    mode = (int(rng.integers(0, 2)), int(rng.integers(0, 2)))
    w = wl.student_random(f"random-large-{seed}", seed, N=N, H=H, W=W, view=k, T=T, n_walls=n_walls,
                          max_steps=max_steps)
    odd = rng.random(w.actions.shape) < 0.05
    w.actions[odd] = rng.integers(-128, 128, size=int(odd.sum()), dtype=np.int8)
    note(f"{w.name}: N={N} {H}x{W} k={k} T={T} max_steps={max_steps} walls={n_walls} mode={mode}")
    env, o = gpu_student(w), cpu_student(w)
    env.set_obs_mode(*mode)
    o.set_obs_mode(*mode)
    cut = int(rng.integers(1, T))
    acts = to_gpu(w.actions)
    out1, out2 = env.step(acts[:cut].contiguous()), env.step(acts[cut:].contiguous())
    torch.cuda.synchronize()
    ref = o.step(w.actions, T)
    assert_rollout_equal(out1, tuple(x[:cut] for x in ref), w.name + " (first call)")
    assert_rollout_equal(out2, tuple(x[cut:] for x in ref), w.name + " (second call)")
    assert_state_equal(env, o)


@pytest.mark.parametrize("seed", range(5000, 5016))
def test_editor_random_shape(seed):
    rng = np.random.default_rng(seed)
    H, W = int(rng.integers(1, 41)), int(rng.integers(1, 41))
    if H * W < 2:
        H = 2
    N = int(rng.choice([1, 63, 128, 129, 300]))
    n_walls = int(rng.integers(0, 2 * H * W))
    ew = wl.editor_random(f"random-editor-{seed}", seed, N, H=H, W=W, n_walls=n_walls)
    extra = int(rng.integers(0, 4))                     # steps past the end of the episode
    T = n_walls + 2 + extra
    actions = rng.integers(-3, H * W + 3, size=(T, N)).astype(np.int32)   # some out of range: clamped
    note(f"{ew.name}: N={N} {H}x{W} walls={n_walls} T={T}")
    ed = binding.EditorEnv(N, H, W, n_walls, device=DEV)
    ed.reset(to_gpu(ew.agent_dir_init))
    obs, t, done = ed.step(to_gpu(actions))
    walls, axy, adir, gxy = ed.get_levels()
    torch.cuda.synchronize()
    oe = oracle.EditorOracle(N, H, W, n_walls)
    oe.reset(ew.agent_dir_init)
    oobs, ot, odone = oe.step(actions, T)
    lv = oe.get_levels()
    assert (obs.cpu().numpy() == oobs).all(), "editor observations differ"
    assert (t.cpu().numpy() == ot).all() and (done.cpu().numpy() == odone).all()
    assert (walls.cpu().numpy() == lv.walls).all() and (axy.cpu().numpy() == lv.agent_xy).all()
    assert (adir.cpu().numpy() == lv.agent_dir).all() and (gxy.cpu().numpy() == lv.goal_xy).all()
